"""Seeded synthetic inputs for shared-prompt attention (Section 4.3 of the paper).

This module only draws numbers and describes shapes: packed
``[prompt | resp_1 | ... | resp_G]`` token layouts (Section 4.3, modification 1),
the head geometry of the model families the paper trains, and N(0,1) values.
It holds none of the attention arithmetic, so both the CPU oracle's tests and
the HIP path can be fed from it without sharing any of the method's code.

The shapes stand in for the paper's GRPO workloads (32 answers per prompt,
16 rollouts sharing a prompt per micro-batch, 1K-16K contexts, bf16
activations); no dataset item is reproduced here.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import torch

_MASK64 = (1 << 64) - 1


class SplitMix64:
    """The public-domain splitmix64 counter generator (Steele, Lea, Flood 2014)."""

    def __init__(self, seed: int):
        self.state = seed & _MASK64

    def next(self) -> int:
        self.state = (self.state + 0x9E3779B97F4A7C15) & _MASK64
        z = self.state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
        return z ^ (z >> 31)


def ragged_lengths(seed: int, count: int, lo: int, hi: int) -> List[int]:
    """``count`` integers uniform in [lo, hi] from a splitmix64 stream."""
    rng = SplitMix64(seed)
    span = hi - lo + 1
    return [lo + (rng.next() % span) for _ in range(count)]


@dataclass
class Group:
    """One prompt with its G responses, in packed order."""
    prompt_len: int
    resp_lens: List[int]

    @property
    def total(self) -> int:
        return self.prompt_len + sum(self.resp_lens)


@dataclass
class Workload:
    """A batch of independent groups packed back to back, plus head geometry."""
    name: str
    groups: List[Group]
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: torch.dtype
    seed: int
    backward: bool = True
    stress_k_fraction: float = 0.0   # fraction of K rows multiplied by stress_k_scale
    stress_k_scale: float = 1.0
    n_sets: int = 1                  # independent q/k/v sets (policy / old / reference)
    scale: Optional[float] = None

    @property
    def total_tokens(self) -> int:
        return sum(g.total for g in self.groups)

    @property
    def softmax_scale(self) -> float:
        return self.scale if self.scale is not None else self.head_dim ** -0.5

    def prompt_lens(self) -> List[int]:
        return [g.prompt_len for g in self.groups]

    def Gs(self) -> List[int]:
        return [len(g.resp_lens) for g in self.groups]

    def resp_lens_flat(self) -> List[int]:
        return [x for g in self.groups for x in g.resp_lens]


def allowed_pairs(group: Group) -> int:
    """Count of (query, key) pairs a group's mask admits: the three terms of the
    complexity split in Section 4.3 (prompt self-attention, response-to-prompt,
    response self-attention), each counted exactly with the diagonal included."""
    lp = group.prompt_len
    n = lp * (lp + 1) // 2
    for li in group.resp_lens:
        n += li * lp + li * (li + 1) // 2
    return n


def useful_flops(w: Workload, backward: bool) -> float:
    """Mask-counted FLOPs: 2 contractions forward (4*d per pair per q head),
    5 backward (10*d per pair per q head)."""
    pairs = sum(allowed_pairs(g) for g in w.groups)
    per_pair = (10 if backward else 4) * w.head_dim
    return float(per_pair) * pairs * w.n_q_heads * w.n_sets


def config(idx: int) -> Workload:
    """The five benchmark configurations (1-based) and two more workloads of many short groups."""
    if idx == 1:
        return Workload("c1_tiny_fp32", [Group(64, [32] * 4)], 2, 2, 64, torch.float32, 1000)
    if idx == 2:
        return Workload("c2_single_group", [Group(1024, [256] * 8)], 28, 4, 128, torch.bfloat16, 2000)
    if idx == 3:
        groups = [Group(4096, ragged_lengths(3000 + g, 16, 128, 512)) for g in range(4)]
        return Workload("c3_long_prompt_ragged", groups, 32, 8, 128, torch.bfloat16, 3000)
    if idx == 4:
        groups = [Group(2048, [1024] * 8) for _ in range(8)]
        return Workload("c4_tri_model_fwd", groups, 28, 4, 128, torch.bfloat16, 4000,
                        backward=False, n_sets=3)
    if idx == 5:
        groups = [Group(16384, ragged_lengths(5000, 32, 64, 256))]
        return Workload("c5_extreme_sharing", groups, 40, 8, 128, torch.bfloat16, 5000,
                        stress_k_fraction=0.01, stress_k_scale=8.0)
    if idx == 6:
        # The shape of the paper's own shared-prompt experiment (Table 3: a 7B model of the Qwen2.5 family,
        # grade-school maths prompts, 1K context per sample, 16 of the 32 rollouts of a prompt in one
        # micro-batch): many groups, each a short prompt and 16 responses of a few hundred tokens.
        # Lengths are seeded stand-ins for that distribution, not dataset items.
        groups = []
        for g in range(64):
            lp = ragged_lengths(6000 + g, 1, 64, 192)[0]
            groups.append(Group(lp, ragged_lengths(6500 + g, 16, 96, 416)))
        return Workload("c6_table3_shape", groups, 28, 4, 128, torch.bfloat16, 6000)
    if idx == 7:
        # 64 groups of 1000 tokens: a prompt of about 70 % and four ragged responses (short-group regime)
        groups = []
        for g in range(64):
            lens = ragged_lengths(9000 + g, 4, 40, 111)
            groups.append(Group(1000 - sum(lens), lens))
        return Workload("c7_short_groups_64x1000", groups, 32, 8, 128, torch.bfloat16, 7000)
    raise ValueError(f"no config {idx}")


def small_ragged(seed: int = 7, dtype: torch.dtype = torch.bfloat16, head_dim: int = 128,
                 n_q_heads: int = 4, n_kv_heads: int = 2,
                 groups: Optional[Sequence[Group]] = None) -> Workload:
    """A workload small enough for a full-tensor oracle comparison that still
    spans several tiles and has ragged tails."""
    if groups is None:
        groups = [Group(333, [1, 63, 65, 0, 127, 129, 200]), Group(70, [300, 5])]
    return Workload(f"small_ragged_{seed}", list(groups), n_q_heads, n_kv_heads, head_dim,
                    dtype, seed)


@dataclass
class Tensors:
    """Host tensors of one q/k/v set: q, d_o are [T, Hq, d]; k, v are [T, Hkv, d]."""
    q: torch.Tensor
    k: torch.Tensor
    v: torch.Tensor
    d_o: Optional[torch.Tensor]
    stressed_rows: List[int] = field(default_factory=list)


def make_tensors(w: Workload, set_index: int = 0) -> Tensors:
    """Draw q, k, v, dO (in that order) ~ N(0,1) in fp32 from a CPU generator seeded
    ``w.seed + set_index``, apply the large-logit stress to K rows if asked, then
    round to ``w.dtype`` (round-to-nearest-even for bf16)."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(w.seed + set_index)
    T, Hq, Hkv, d = w.total_tokens, w.n_q_heads, w.n_kv_heads, w.head_dim
    q = torch.randn(T, Hq, d, generator=gen, dtype=torch.float32)
    k = torch.randn(T, Hkv, d, generator=gen, dtype=torch.float32)
    v = torch.randn(T, Hkv, d, generator=gen, dtype=torch.float32)
    d_o = torch.randn(T, Hq, d, generator=gen, dtype=torch.float32) if w.backward else None
    stressed: List[int] = []
    if w.stress_k_fraction > 0.0:
        pick = torch.rand(T, generator=gen) < w.stress_k_fraction
        k[pick] *= w.stress_k_scale
        stressed = torch.nonzero(pick).flatten().tolist()
    cast = lambda x: None if x is None else x.to(w.dtype).contiguous()
    return Tensors(cast(q), cast(k), cast(v), cast(d_o), stressed)


def make_tensors_on_device(w: Workload, device) -> Tensors:
    """The same recipe drawn by the device's generator (seed ``w.seed``; q, k, v, dO in that
    order, N(0,1) rounded to ``w.dtype``), for packings whose tensors are several GiB each and
    would take minutes to draw on the host.  A consumer that needs host values copies the
    slices it wants from these tensors."""
    gen = torch.Generator(device=device)
    gen.manual_seed(w.seed)
    T, Hq, Hkv, d = w.total_tokens, w.n_q_heads, w.n_kv_heads, w.head_dim

    def draw(heads):
        return torch.empty(T, heads, d, dtype=w.dtype, device=device).normal_(generator=gen)

    q, k, v = draw(Hq), draw(Hkv), draw(Hkv)
    return Tensors(q, k, v, draw(Hq) if w.backward else None)
