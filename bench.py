#!/usr/bin/env python3
"""Benchmark of the shared-prompt attention hot path on one MI355X.

A "step" is one forward (O, LSE) plus one backward (D, dK/dV pass, dQ pass) of the
headline workload: config 5, the largest long-prompt configuration (one group,
prompt 16384, 32 ragged responses, 40 q / 8 kv heads, head_dim 128, bf16).  Inputs are
seeded synthetic tensors already resident in HBM.  `value` is useful (mask-counted)
TFLOP/s over forward+backward; forward-only and backward-only rates, each stage's mean
duration (HIP events on the launch stream, inside the timed region) and the roofline of
the dominant kernel are reported beside it, with the CPU oracle timed on a bounded
sample of the same workload.

usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 5] [--no-cpu]
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA peak


def parse_traffic(workload: str, kernel: str):
    """HBM bytes per launch of `kernel`, taken from the committed rocprofv3 --pmc summary
    (FETCH_SIZE + WRITE_SIZE, scaled by the copy-kernel calibration); None if absent."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}.txt")
    if not os.path.exists(path):
        return None
    pat = re.compile(rf"^{re.escape(kernel)}\s+hbm_bytes_per_launch\s+([0-9.eE+]+)")
    with open(path) as f:
        for line in f:
            m = pat.match(line.strip())
            if m:
                return float(m.group(1))
    return None


def cpu_baseline(w, t, target_seconds=12.0):
    """Time the fp64 oracle (as it stands) on whole q heads of the workload's first group:
    forward and backward (forward only for a forward-only workload) over all rows of each head, one
    head at a time until about `target_seconds` of CPU work has been done.  Useful FLOPs per head =
    14 * d * pairs (4 * d * pairs forward only)."""
    import numpy as np
    from oracle import sp_attn_oracle as orc
    from paper_2511_18871_amd import workloads as W
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    g = w.groups[0]
    n = g.total
    sl = slice(0, n)
    rep = w.n_q_heads // w.n_kv_heads
    heads, dt = 0, 0.0
    while heads < w.n_q_heads and dt < target_seconds:
        t0 = time.perf_counter()
        if w.backward:      # the oracle's backward recomputes the forward: 4*d + 10*d FLOPs per pair
            orc.sp_attn_bwd(t.q[sl], t.k[sl], t.v[sl], t.d_o[sl], g.prompt_len, g.resp_lens, w.softmax_scale,
                            kv_heads=[heads // rep], q_heads=[heads], row_block=1024)
        else:
            orc.sp_attn_fwd(t.q[sl], t.k[sl], t.v[sl], g.prompt_len, g.resp_lens, w.softmax_scale,
                            heads=[heads], row_block=1024)
        dt += time.perf_counter() - t0
        heads += 1
    flops = (14.0 if w.backward else 4.0) * w.head_dim * W.allowed_pairs(g) * heads
    passes = "forward+backward" if w.backward else "forward"
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": f"q heads 0..{heads - 1} of {w.n_q_heads}, all {n} rows of group 0, {passes} in "
                      f"fp64, {dt:.1f} s",
            "seconds": dt}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=5)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline leg")
    ap.add_argument("--no-naive", action="store_true", help="skip the naive packed-causal forward baseline")
    ap.add_argument("--no-ceiling", action="store_true", help="skip the MFMA-only ceiling loops")
    ap.add_argument("--small-steps", type=int, default=-1,
                    help="override the library's threshold for the 128-row kernel shape (0: always 256 rows)")
    ap.add_argument("--inputs", choices=["random", "zeros"], default="random",
                    help="zeros: run the same kernels on all-zero tensors (a power diagnostic: the instruction\n"
                         "stream is identical, only operand toggling differs; not the metric)")
    ap.add_argument("--response-rows", action="store_true",
                    help="also time forward and backward restricted to response rows (a later micro-batch of a\n"
                         "prompt whose prompt rows were already computed)")
    ap.add_argument("--loss", action="store_true",
                    help="also time the response-token log-probability forward/backward and the GRPO objective\n"
                         "over logits [T, 151936] generated on the device")
    ap.add_argument("--rope", action="store_true",
                    help="also time the rotary-embedding pass (restarted positions) over q and k")
    ap.add_argument("--cold", action="store_true",
                    help="overwrite a 1 GiB buffer before every step so that L2 and the Infinity Cache hold none of "
                         "the inputs; throughput is then taken from the summed stage times, not the wall clock")
    ap.add_argument("--no-reserve", action="store_true",
                    help="give the calls a workspace without room for the forward-to-backward reserve (the backward then "
                         "forms D from the bf16 o alone): measures what the reserve costs")
    ap.add_argument("--probe-atomics", action="store_true",
                    help="also measure the fp32 atomic-add rate that a one-pass backward's dQ accumulation would need")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 1 GiB device copy (counter calibration for rocprofv3 --pmc runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2511_18871_amd import binding as B
    from paper_2511_18871_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    B.load_library()
    B.set_small_shape_steps(args.small_steps)
    w = W.config(args.config)
    dev = torch.device("cuda:0")
    if w.total_tokens * w.n_q_heads > 4_000_000:
        # tensors of a GiB and more are drawn by the device's generator (same recipe); the CPU leg copies
        # the first group's slice back
        t = W.make_tensors_on_device(w, dev)
        q, k, v, d_o = t.q, t.k, t.v, t.d_o
        n0 = w.groups[0].total
        t = W.Tensors(q[:n0].cpu(), k[:n0].cpu(), v[:n0].cpu(), None if d_o is None else d_o[:n0].cpu())
    else:
        t = W.make_tensors(w)
        q, k, v = t.q.to(dev), t.k.to(dev), t.v.to(dev)
        d_o = t.d_o.to(dev) if t.d_o is not None else None
    if args.inputs == "zeros":
        q, k, v = torch.zeros_like(q), torch.zeros_like(k), torch.zeros_like(v)
        d_o = torch.zeros_like(d_o) if d_o is not None else None
    pl, Gs, rl = w.prompt_lens(), w.Gs(), w.resp_lens_flat()
    scale = w.softmax_scale
    T, Hq, Hkv, d = w.total_tokens, w.n_q_heads, w.n_kv_heads, w.head_dim
    code = B.SP_BF16 if w.dtype == torch.bfloat16 else B.SP_F32
    o = torch.empty_like(q)
    lse = torch.empty(Hq, T, dtype=torch.float32, device=dev)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    # one workspace for the forward and the backward, with room for the forward-to-backward reserve
    ws = torch.empty(B.workspace_bytes(True, T, len(pl), len(rl), Hq, Hkv, d, code)
                     + (0 if args.no_reserve else B.reserve_bytes(T, Hq, d, code)), dtype=torch.uint8, device=dev)
    do_bwd = w.backward

    # the backward as two stage calls (what one sp_attn_bwd_batched call runs, split so that each pass can be
    # timed): the rowsum and dq stages together (the bf16 dq pass forms D itself), then the dkdv pass
    stage_names = ["fwd"] + (["bwd_rowsum_dq", "bwd_dkdv"] if do_bwd else [])

    def step(events=None):
        def mark(i):
            if events is not None:
                events[i].record()
        mark(0)
        B.sp_attn_fwd_batched(q, k, v, pl, Gs, rl, scale, o=o, lse=lse, workspace=ws)
        mark(1)
        if do_bwd:
            B.sp_attn_bwd_batched_stages(q, k, v, o, lse, d_o, pl, Gs, rl, scale,
                                         B.SP_BWD_STAGE_ROWSUM | B.SP_BWD_STAGE_DQ, ws, dq=dq)
            mark(2)
            B.sp_attn_bwd_batched_stages(q, k, v, None, lse, d_o, pl, Gs, rl, scale, B.SP_BWD_STAGE_DKDV, ws,
                                         dk=dk, dv=dv)
            mark(3)

    flush = torch.empty(1 << 30, dtype=torch.uint8, device=dev) if args.cold else None
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    n_ev = len(stage_names) + 1
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(n_ev)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        if flush is not None:
            flush.fill_(i & 0xFF)
        step(evs[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    stage_ms = {}
    for si, name in enumerate(stage_names):
        stage_ms[name] = sum(evs[i][si].elapsed_time(evs[i][si + 1]) for i in range(args.steps)) / args.steps
    # per-step GPU time (sum of the stage event intervals of that step): median and minimum over the steps
    per_step = sorted(sum(evs[i][si].elapsed_time(evs[i][si + 1]) for si in range(len(stage_names)))
                      for i in range(args.steps))
    step_median = per_step[len(per_step) // 2] if len(per_step) % 2 else 0.5 * (per_step[len(per_step) // 2 - 1] + per_step[len(per_step) // 2])
    if flush is not None:
        ms_per_step = sum(stage_ms.values())

    fwd_flops = W.useful_flops(w, False) / w.n_sets
    bwd_flops = W.useful_flops(w, True) / w.n_sets if do_bwd else 0.0
    total_flops = fwd_flops + bwd_flops
    value = total_flops / (ms_per_step * 1e-3) / 1e12
    fwd_tf = fwd_flops / (stage_ms["fwd"] * 1e-3) / 1e12

    out = {
        "metric": "shared-prompt attn fwd+bwd useful TFLOP/s and % bf16 MFMA peak, 1xMI355X",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == torch.bfloat16 else "f32",
        "data": "synthetic" if args.inputs == "random" else "all-zero tensors (power diagnostic, not the metric)",
        "config": {"workload": w.name, "groups": len(w.groups), "prompt_len": w.groups[0].prompt_len,
                   "G": len(w.groups[0].resp_lens), "total_tokens": T, "n_q_heads": Hq, "n_kv_heads": Hkv,
                   "head_dim": d, "passes": "fwd+bwd" if do_bwd else "fwd"},
        "pct_peak": round(100.0 * value / PEAK_BF16_TFLOPS, 2),
        "fwd": {"ms": round(stage_ms["fwd"], 4), "tflops": round(fwd_tf, 2),
                "pct_peak": round(100.0 * fwd_tf / PEAK_BF16_TFLOPS, 2)},
        "stage_ms": {k_: round(v_, 4) for k_, v_ in stage_ms.items()},
        "step_gpu_ms": {"median": round(step_median, 4), "min": round(per_step[0], 4), "max": round(per_step[-1], 4)},
    }
    if flush is not None:
        out["cold_cache"] = True
    if args.no_reserve:
        out["reserve"] = False
    if do_bwd:
        bwd_ms = stage_ms["bwd_rowsum_dq"] + stage_ms["bwd_dkdv"]
        bwd_tf = bwd_flops / (bwd_ms * 1e-3) / 1e12
        out["bwd"] = {"ms": round(bwd_ms, 4), "tflops": round(bwd_tf, 2),
                      "pct_peak": round(100.0 * bwd_tf / PEAK_BF16_TFLOPS, 2)}
        # dominant kernel: the dkdv pass.  Algorithmic FLOPs per launch: its four contractions
        # (S, dP, dV, dK) are all required for dK/dV = 8*d per allowed pair per q head.
        dk_flops = 0.8 * bwd_flops
        ach = dk_flops / (stage_ms["bwd_dkdv"] * 1e-3) / 1e12
        out["roofline"] = {"kernel": "bwd_dkdv_kernel", "bound": "mfma", "achieved": round(ach, 2),
                           "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(ach / PEAK_BF16_TFLOPS, 4),
                           "traffic": parse_traffic(w.name, "bwd_dkdv_kernel")}
    else:
        out["roofline"] = {"kernel": "fwd_kernel", "bound": "mfma", "achieved": round(fwd_tf, 2),
                           "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(fwd_tf / PEAK_BF16_TFLOPS, 4),
                           "traffic": parse_traffic(w.name, "fwd_kernel")}
    out["roofline_fwd"] = {"kernel": "fwd_kernel", "bound": "mfma", "achieved": round(fwd_tf, 2),
                           "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(fwd_tf / PEAK_BF16_TFLOPS, 4),
                           "traffic": parse_traffic(w.name, "fwd_kernel")}

    if w.dtype == torch.bfloat16 and not args.no_naive:
        # naive packed-causal baseline: the same kernel visiting every tile at or below the diagonal of the
        # packed sequence with an element-wise mask; useful FLOPs in the numerator, like the product path
        evn = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        B.sp_attn_fwd_batched(q, k, v, pl, Gs, rl, scale, schedule=B.SP_SCHED_NAIVE_CAUSAL, o=o, lse=lse, workspace=ws)
        evn[0].record()
        for _ in range(5):
            B.sp_attn_fwd_batched(q, k, v, pl, Gs, rl, scale, schedule=B.SP_SCHED_NAIVE_CAUSAL, o=o, lse=lse,
                                  workspace=ws)
        evn[1].record()
        torch.cuda.synchronize()
        nms = evn[0].elapsed_time(evn[1]) / 5
        out["naive_fwd"] = {"ms": round(nms, 4), "useful_tflops": round(fwd_flops / (nms * 1e-3) / 1e12, 2),
                            "speedup_of_shared_schedule": round(nms / stage_ms["fwd"], 3)}

    if w.dtype == torch.bfloat16 and not args.no_ceiling:
        # what a loop of nothing but bf16 MFMAs sustains on this machine, per LDS operands read per MFMA and per
        # operand values (N(0,1) like the workload's tensors; all-ones for the same loop at low power)
        gen = torch.Generator(device="cpu").manual_seed(7)
        n_op = 8 * 512 * 8
        rnd = [torch.randn(n_op, generator=gen).to(torch.bfloat16).to(dev) for _ in range(2)]
        one = [torch.ones(n_op, dtype=torch.bfloat16, device=dev) for _ in range(2)]
        sink = torch.empty(512, dtype=torch.float32, device=dev)
        ceil = {}
        for data_name, (xa, xb) in (("random", rnd), ("ones", one)):
            for n_lds in (0, 1, 2):
                B.sp_attn_mfma_ceiling(n_lds, xa, xb, 200, sink)
                evc = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
                evc[0].record()
                fl = B.sp_attn_mfma_ceiling(n_lds, xa, xb, 6000, sink)      # about 3 ms: long enough to settle the clock
                evc[1].record()
                torch.cuda.synchronize()
                ceil[f"{data_name}_lds{n_lds}"] = round(fl / (evc[0].elapsed_time(evc[1]) * 1e-3) / 1e12, 1)
        out["mfma_ceiling"] = {"unit": "TFLOP/s", **ceil,
                               "note": "bf16 32x32x16 MFMA loop, 8 waves per CU; ldsN = operands read from LDS per MFMA"}
        # the attention kernels against the ceiling of their own operand mix on random data
        out["fwd"]["pct_of_measured_ceiling"] = round(100.0 * fwd_tf / ceil["random_lds1"], 1)
        if do_bwd:
            # executed rates: the dq pass (timed with the rowsum folded in and the edge kernel) runs 6*d and the dkdv pass 8*d FLOPs
            # per allowed pair and q head
            pairs_hq = fwd_flops / (4.0 * d)
            dq_exec = 6.0 * d * pairs_hq / (stage_ms["bwd_rowsum_dq"] * 1e-3) / 1e12
            dkdv_exec = 8.0 * d * pairs_hq / (stage_ms["bwd_dkdv"] * 1e-3) / 1e12
            out["bwd"]["dq_executed_tflops"] = round(dq_exec, 1)
            out["bwd"]["dkdv_executed_tflops"] = round(dkdv_exec, 1)
            out["bwd"]["dq_pct_of_measured_ceiling"] = round(100.0 * dq_exec / ceil["random_lds1"], 1)
            out["bwd"]["dkdv_pct_of_measured_ceiling"] = round(
                100.0 * dkdv_exec / (0.5 * (ceil["random_lds1"] + ceil["random_lds2"])), 1)

    if w.n_sets > 1:
        # all weight sets of the workload (policy / old policy / reference) in one launch,
        # beside n_sets separate launches of the same kernel
        sets = [t] + [W.make_tensors(w, i) for i in range(1, w.n_sets)]
        qs, ks, vs = [x.q.to(dev) for x in sets], [x.k.to(dev) for x in sets], [x.v.to(dev) for x in sets]
        os_ = [torch.empty_like(x) for x in qs]
        ls_ = [torch.empty(Hq, T, dtype=torch.float32, device=dev) for _ in qs]
        evm = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        B.sp_attn_fwd_multi(qs, ks, vs, pl, Gs, rl, scale, os=os_, lses=ls_, workspace=ws)
        evm[0].record()
        for _ in range(5):
            B.sp_attn_fwd_multi(qs, ks, vs, pl, Gs, rl, scale, os=os_, lses=ls_, workspace=ws)
        evm[1].record()
        for _ in range(5):
            for i in range(w.n_sets):
                B.sp_attn_fwd_batched(qs[i], ks[i], vs[i], pl, Gs, rl, scale, o=os_[i], lse=ls_[i], workspace=ws)
        evm[2].record()
        torch.cuda.synchronize()
        mms, sms = evm[0].elapsed_time(evm[1]) / 5, evm[1].elapsed_time(evm[2]) / 5
        out["multi_set_fwd"] = {"sets": w.n_sets, "one_launch_ms": round(mms, 4), "separate_launches_ms": round(sms, 4),
                                "tflops": round(fwd_flops * w.n_sets / (mms * 1e-3) / 1e12, 2)}

    if args.response_rows and do_bwd:
        fl = B.SP_FLAG_RESPONSE_ROWS
        evq = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        B.sp_attn_fwd_batched_ex(q, k, v, pl, Gs, rl, scale, fl, o=o, lse=lse, workspace=ws)
        B.sp_attn_bwd_batched_ex(q, k, v, o, lse, d_o, pl, Gs, rl, scale, fl | B.SP_FLAG_ACCUMULATE_DKDV, dq=dq, dk=dk,
                                 dv=dv, workspace=ws)
        evq[0].record()
        for _ in range(5):
            B.sp_attn_fwd_batched_ex(q, k, v, pl, Gs, rl, scale, fl, o=o, lse=lse, workspace=ws)
        evq[1].record()
        for _ in range(5):
            B.sp_attn_bwd_batched_ex(q, k, v, o, lse, d_o, pl, Gs, rl, scale, fl | B.SP_FLAG_ACCUMULATE_DKDV, dq=dq,
                                     dk=dk, dv=dv, workspace=ws)
        evq[2].record()
        torch.cuda.synchronize()
        # pairs whose query is a response row (terms B and C of the section's complexity split)
        pairs_all = sum(W.allowed_pairs(g) for g in w.groups)
        pairs_resp = pairs_all - sum(g.prompt_len * (g.prompt_len + 1) // 2 for g in w.groups)
        fms, bms = evq[0].elapsed_time(evq[1]) / 5, evq[1].elapsed_time(evq[2]) / 5
        rf = 4.0 * d * pairs_resp * Hq
        out["response_rows"] = {"pair_fraction": round(pairs_resp / pairs_all, 4), "fwd_ms": round(fms, 4),
                                "bwd_ms": round(bms, 4), "fwd_tflops": round(rf / (fms * 1e-3) / 1e12, 2),
                                "bwd_tflops": round(2.5 * rf / (bms * 1e-3) / 1e12, 2)}
        # the buffers were overwritten / accumulated into: restore nothing, the timed steps are done

    if args.loss:
        # HBM-bound passes over the response rows of logits [T, V] (V = the Qwen2.5 vocabulary)
        V = 151936
        gen = torch.Generator(device=dev).manual_seed(w.seed)
        z = torch.randn(T, V, generator=gen, device=dev, dtype=torch.float32).mul_(2.0).to(torch.bfloat16)
        yl = torch.randint(0, V, (T,), generator=gen, device=dev, dtype=torch.int32)
        dz = torch.empty_like(z)
        n_resp_tok = sum(rl)
        adv = torch.randn(len(rl), generator=gen, device=dev)
        logp, lsev = B.sp_attn_logprob_fwd(z, yl, pl, Gs, rl)
        old_lp = logp + 0.1 * torch.randn(T, generator=gen, device=dev)
        evl = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        evl[0].record()
        for _ in range(5):
            B.sp_attn_logprob_fwd(z, yl, pl, Gs, rl, logp=logp, lse=lsev)
        evl[1].record()
        for _ in range(5):
            _, gl = B.sp_attn_grpo_loss(logp, old_lp, old_lp, adv, pl, Gs, rl)
        evl[2].record()
        for _ in range(5):
            B.sp_attn_logprob_bwd(z, yl, lsev, gl, pl, Gs, rl, dlogits=dz)
        evl[3].record()
        torch.cuda.synchronize()
        fms, gms, bms = (evl[i].elapsed_time(evl[i + 1]) / 5 for i in range(3))
        fb, bb = n_resp_tok * V * 2, 2 * n_resp_tok * V * 2
        out["loss"] = {"vocab": V, "response_tokens": n_resp_tok,
                       "logprob_fwd": {"ms": round(fms, 4), "bytes": fb, "achieved": round(fb / (fms * 1e-3) / 1e9, 1)},
                       "logprob_bwd": {"ms": round(bms, 4), "bytes": bb, "achieved": round(bb / (bms * 1e-3) / 1e9, 1)},
                       "grpo_ms": round(gms, 4), "bound": "hbm", "peak": 8000.0, "unit": "GB/s"}
        del z, dz

    if args.rope:
        # HBM-bound pass: reads and writes q [T,Hq,d] and k [T,Hkv,d] once each; one launch for both, beside
        # one launch per tensor
        qr, kr = torch.empty_like(q), torch.empty_like(k)
        evr = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        B.sp_attn_rope_qk(q, k, pl, Gs, rl, 1e6, q_out=qr, k_out=kr, workspace=ws)
        evr[0].record()
        for _ in range(10):
            B.sp_attn_rope_qk(q, k, pl, Gs, rl, 1e6, q_out=qr, k_out=kr, workspace=ws)
        evr[1].record()
        for _ in range(10):
            B.sp_attn_rope(q, pl, Gs, rl, 1e6, out=qr, workspace=ws)
            B.sp_attn_rope(k, pl, Gs, rl, 1e6, out=kr, workspace=ws)
        evr[2].record()
        torch.cuda.synchronize()
        rms, rms2 = evr[0].elapsed_time(evr[1]) / 10, evr[1].elapsed_time(evr[2]) / 10
        nbytes = 2 * (q.numel() + k.numel()) * q.element_size()
        out["rope"] = {"ms": round(rms, 4), "two_launches_ms": round(rms2, 4), "bytes": nbytes, "bound": "hbm",
                       "achieved": round(nbytes / (rms * 1e-3) / 1e9, 1), "peak": 8000.0, "unit": "GB/s",
                       "frac": round(nbytes / (rms * 1e-3) / 8e12, 4)}

    if args.probe_atomics:
        # the one-pass backward's dQ accumulation, alone: fp32 atomic adds of 64 x 128 tiles into [T, Hq, 128]
        rows = (T + 63) // 64 * 64
        acc = torch.zeros(rows * Hq * 128, dtype=torch.float32, device=dev)
        res = {}
        for name, layout in (("row_contiguous", 0), ("accumulator_scatter", 1)):
            B.sp_attn_probe_atomic_add(acc, rows, Hq, 20, layout=layout)
            eva = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            eva[0].record()
            nb = B.sp_attn_probe_atomic_add(acc, rows, Hq, 1000 if layout == 0 else 200, layout=layout)
            eva[1].record()
            torch.cuda.synchronize()
            res[name] = round(nb / (eva[0].elapsed_time(eva[1]) * 1e-3) / 1e9, 1)
        pairs_hq = fwd_flops / (4.0 * d)
        need = 4.0 * pairs_hq
        out["atomic_add_probe"] = {"unit": "GB/s", **res, "one_pass_dq_bytes": need,
                                   "one_pass_dq_ms_at_best_rate": round(need / (max(res.values()) * 1e9) * 1e3, 2),
                                   "note": "fp32 atomic adds a one-pass backward would issue for dQ (4 bytes per allowed "
                                           "pair and q head) against this box's measured rate; the dq pass takes "
                                           f"{stage_ms.get('bwd_rowsum_dq', 0.0):.2f} ms"}
        del acc

    if args.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        out["calib_copy_bytes"] = 1 << 30

    if not args.no_cpu:
        out["cpu_baseline"] = {k_: (round(v_, 6) if isinstance(v_, float) else v_)
                               for k_, v_ in cpu_baseline(w, t).items()}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
