"""GPU parity on seeded random packings: group counts, prompt lengths, response counts and lengths
drawn so that tile edges, empty segments, ragged tails and the padded tail of the key loop are hit
in many combinations.  Every tensor is compared element by element with the fp64 oracle."""
import numpy as np
import pytest
import torch

from paper_2511_18871_amd import binding as B
from paper_2511_18871_amd import workloads as W
from parity import gate, gate_lse, oracle_bwd, to64

pytestmark = pytest.mark.gpu

HEADS = [(4, 2), (6, 2), (8, 8), (5, 1), (2, 1)]


def random_workload(seed):
    rng = np.random.default_rng(1000 + seed)
    groups = []
    for _ in range(int(rng.integers(1, 4))):
        lp = int(rng.choice([0, 1, 63, 64, 65, 127, 255, 256, 257, int(rng.integers(2, 700))]))
        G = int(rng.integers(0, 7))
        lens = [int(rng.choice([0, 1, 31, 32, 33, 64, int(rng.integers(1, 300))])) for _ in range(G)]
        if lp + sum(lens) == 0:
            lp = 1
        groups.append(W.Group(lp, lens))
    hq, hkv = HEADS[seed % len(HEADS)]
    return W.Workload(f"rand{seed}", groups, hq, hkv, 128, torch.bfloat16, 300 + seed)


# 0..13: the first seeds of the generator.  The others are the seeds, of 1500 more drawn once, on which an
# earlier version of the backward missed the max-abs gate by 1-23 % (dQ of rows with two or three keys, dK of
# keys seen by two or three rows: the bf16 rounding of dS did not average out there).
@pytest.mark.parametrize("seed", list(range(14)) + [360, 910, 1190, 1306, 1482])
def test_random_packing_fwd_bwd(seed):
    w = random_workload(seed)
    t = W.make_tensors(w)
    pl, Gs, rl, sc = w.prompt_lens(), w.Gs(), w.resp_lens_flat(), w.softmax_scale
    q, k, v, d_o = t.q.cuda(), t.k.cuda(), t.v.cuda(), t.d_o.cuda()
    o, lse = B.sp_attn_fwd_batched(q, k, v, pl, Gs, rl, sc)
    dq, dk, dv = B.sp_attn_bwd_batched(q, k, v, o, lse, d_o, pl, Gs, rl, sc)
    torch.cuda.synchronize()
    rdq, rdk, rdv, ro, rlse = oracle_bwd(w, t)
    desc = f"{[(g.prompt_len, g.resp_lens) for g in w.groups]} heads {w.n_q_heads}/{w.n_kv_heads}"
    gate("O " + desc, to64(o), ro, w.dtype)
    gate_lse(to64(lse), rlse, w.dtype)
    gate("dQ " + desc, to64(dq), rdq, w.dtype)
    gate("dK " + desc, to64(dk), rdk, w.dtype)
    gate("dV " + desc, to64(dv), rdv, w.dtype)


# Both workgroup shapes of the forward and of the dq pass (256 rows, whole 64-key tiles; 128 rows, half tiles, two
# workgroups per CU), each forced on packings the library would give to the other: a group's last tile may end
# in its first half, so that the 128-row shape's copy of the second half lies wholly past the group's end.
@pytest.mark.parametrize("steps", [0, 1 << 20])
@pytest.mark.parametrize("seed", [2, 5, 11, 360, 1306])
def test_random_packing_both_workgroup_shapes(seed, steps):
    try:
        B.set_small_shape_steps(steps)
        test_random_packing_fwd_bwd(seed)
    finally:
        B.set_small_shape_steps(-1)


@pytest.mark.parametrize("steps", [0, 1 << 20])
@pytest.mark.parametrize("tail", [1, 31, 32, 33, 63, 64])
def test_group_end_inside_either_half_of_the_last_tile(tail, steps):
    """Group lengths 256 + tail and 128 + tail: the last key tile ends after `tail` keys."""
    groups = [W.Group(200, [56 + tail]), W.Group(0, [128 + tail]), W.Group(64 + tail, [])]
    w = W.Workload(f"tail{tail}", groups, 4, 2, 128, torch.bfloat16, 500 + tail)
    t = W.make_tensors(w)
    pl, Gs, rl, sc = w.prompt_lens(), w.Gs(), w.resp_lens_flat(), w.softmax_scale
    q, k, v, d_o = t.q.cuda(), t.k.cuda(), t.v.cuda(), t.d_o.cuda()
    try:
        B.set_small_shape_steps(steps)
        o, lse = B.sp_attn_fwd_batched(q, k, v, pl, Gs, rl, sc)
        dq, dk, dv = B.sp_attn_bwd_batched(q, k, v, o, lse, d_o, pl, Gs, rl, sc)
        torch.cuda.synchronize()
    finally:
        B.set_small_shape_steps(-1)
    rdq, rdk, rdv, ro, rlse = oracle_bwd(w, t)
    gate("O", to64(o), ro, w.dtype)
    gate_lse(to64(lse), rlse, w.dtype)
    gate("dQ", to64(dq), rdq, w.dtype)
    gate("dK", to64(dk), rdk, w.dtype)
    gate("dV", to64(dv), rdv, w.dtype)


@pytest.mark.parametrize("heads", [(6, 3), (12, 12), (10, 5), (48, 24)])
def test_kv_head_counts_that_neither_divide_nor_are_a_multiple_of_8(heads):
    """Such head counts take the plain block -> (tile, head) mapping instead of the XCD-aware ones."""
    w = random_workload(3)
    w = W.Workload(f"heads{heads}", w.groups, heads[0], heads[1], 128, torch.bfloat16, 411)
    t = W.make_tensors(w)
    pl, Gs, rl, sc = w.prompt_lens(), w.Gs(), w.resp_lens_flat(), w.softmax_scale
    q, k, v, d_o = t.q.cuda(), t.k.cuda(), t.v.cuda(), t.d_o.cuda()
    o, lse = B.sp_attn_fwd_batched(q, k, v, pl, Gs, rl, sc)
    dq, dk, dv = B.sp_attn_bwd_batched(q, k, v, o, lse, d_o, pl, Gs, rl, sc)
    torch.cuda.synchronize()
    rdq, rdk, rdv, ro, rlse = oracle_bwd(w, t)
    gate("O", to64(o), ro, w.dtype)
    gate_lse(to64(lse), rlse, w.dtype)
    gate("dQ", to64(dq), rdq, w.dtype)
    gate("dK", to64(dk), rdk, w.dtype)
    gate("dV", to64(dv), rdv, w.dtype)
