"""GPU parity on batches of many groups: the tile -> group lookup (bisection on the segment table's
running tile counts), a segment table of several upload launches, and tensors larger than 4 GiB
(element indices beyond 2^31, byte offsets beyond 2^32)."""
import numpy as np
import pytest
import torch

from oracle import rope_oracle, sp_attn_oracle as orc
from paper_2511_18871_amd import binding as B
from paper_2511_18871_amd import workloads as W
from parity import gate, gate_lse, oracle_bwd, to64

pytestmark = pytest.mark.gpu


def many_groups(seed, n_groups, max_prompt, max_g, max_len, heads, dtype, head_dim):
    rng = np.random.default_rng(seed)
    groups = []
    for _ in range(n_groups):
        lp = int(rng.integers(0, max_prompt + 1))
        lens = [int(rng.integers(0, max_len + 1)) for _ in range(int(rng.integers(0, max_g + 1)))]
        if lp + sum(lens) == 0:
            lp = 1
        groups.append(W.Group(lp, lens))
    return W.Workload(f"many{seed}", groups, heads[0], heads[1], head_dim, dtype, 7000 + seed)


@pytest.mark.parametrize("dtype,heads,head_dim,n_groups", [(torch.bfloat16, (4, 2), 128, 300),
                                                          (torch.float32, (2, 1), 64, 120)])
def test_hundreds_of_small_groups_every_element(dtype, heads, head_dim, n_groups):
    w = many_groups(1, n_groups, 280, 3, 140, heads, dtype, head_dim)
    t = W.make_tensors(w)
    pl, Gs, rl, sc = w.prompt_lens(), w.Gs(), w.resp_lens_flat(), w.softmax_scale
    q, k, v, d_o = t.q.cuda(), t.k.cuda(), t.v.cuda(), t.d_o.cuda()
    o, lse = B.sp_attn_fwd_batched(q, k, v, pl, Gs, rl, sc)
    dq, dk, dv = B.sp_attn_bwd_batched(q, k, v, o, lse, d_o, pl, Gs, rl, sc)
    torch.cuda.synchronize()
    rdq, rdk, rdv, ro, rlse = oracle_bwd(w, t)
    print(gate("O", to64(o), ro, dtype))
    gate_lse(to64(lse), rlse, dtype)
    print(gate("dQ", to64(dq), rdq, dtype))
    print(gate("dK", to64(dk), rdk, dtype))
    print(gate("dV", to64(dv), rdv, dtype))


def test_tensors_beyond_4_gib_sampled_groups():
    """1100 groups, 1.1e6 tokens, 32 q / 16 kv heads: q, o, dO, dq are 9 GB each (element index up to
    4.5e9), k, v, dk, dv 4.5 GB each.  Groups are independent, so the oracle on one group's slice
    is the exact expectation for that group's rows; checked for the first and last group and the
    groups that contain the tokens where q's and k's offsets cross 2^31 elements / 2^32 bytes."""
    n_groups, Hq, Hkv, d = 1100, 32, 16, 128
    groups = []
    for g in range(n_groups):
        lens = W.ragged_lengths(9000 + g, 4, 40, 110)
        groups.append(W.Group(1000 - sum(lens), lens))           # 1000 tokens per group, ragged inside
    w = W.Workload("beyond_4gib", groups, Hq, Hkv, d, torch.bfloat16, 9000)
    T = w.total_tokens
    assert T * Hq * d > 2 ** 32 and T * Hkv * d > 2 ** 31
    t = W.make_tensors_on_device(w, torch.device("cuda:0"))
    pl, Gs, rl, sc = w.prompt_lens(), w.Gs(), w.resp_lens_flat(), w.softmax_scale
    o, lse = B.sp_attn_fwd_batched(t.q, t.k, t.v, pl, Gs, rl, sc)
    dq, dk, dv = B.sp_attn_bwd_batched(t.q, t.k, t.v, o, lse, t.d_o, pl, Gs, rl, sc)
    qr = B.sp_attn_rope(t.q, pl, Gs, rl, 1.0e6)
    torch.cuda.synchronize()
    for name, x in (("o", o), ("lse", lse), ("dq", dq), ("dk", dk), ("dv", dv)):
        assert bool(torch.isfinite(x).all()), name

    crossings = [2 ** 31 // (Hq * d), 2 ** 32 // (Hq * d), 2 ** 31 // (Hkv * d), 2 ** 32 // (Hkv * d)]
    picked = sorted({0, n_groups - 1} | {tok // 1000 for tok in crossings if tok < T}
                    | {tok // 1000 + 1 for tok in crossings if tok // 1000 + 1 < n_groups})
    assert len(picked) >= 6
    cpu = lambda x, sl: x[sl].cpu()
    for gi in picked:
        g, sl = groups[gi], slice(1000 * gi, 1000 * (gi + 1))
        qg, kg, vg, gg = cpu(t.q, sl), cpu(t.k, sl), cpu(t.v, sl), cpu(t.d_o, sl)
        rdq, rdk, rdv, ro, rlse = orc.sp_attn_bwd(qg, kg, vg, gg, g.prompt_len, g.resp_lens, sc)
        print(gi, gate(f"O[g{gi}]", to64(o[sl]), ro, w.dtype))
        gate_lse(to64(lse[:, sl]), rlse, w.dtype)
        print(gi, gate(f"dQ[g{gi}]", to64(dq[sl]), rdq, w.dtype))
        print(gi, gate(f"dK[g{gi}]", to64(dk[sl]), rdk, w.dtype))
        print(gi, gate(f"dV[g{gi}]", to64(dv[sl]), rdv, w.dtype))
        ref = rope_oracle.rope_rotate(to64(qg), rope_oracle.positions(g.prompt_len, g.resp_lens), 1.0e6)
        err = np.abs(to64(qr[sl]) - ref)
        assert float(err.max()) <= 2.0 ** -7 * max(1.0, float(np.abs(ref).max())), (gi, float(err.max()))
