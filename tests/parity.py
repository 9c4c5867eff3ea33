"""Helpers shared by the GPU parity tests: tolerance gates and oracle drivers."""
import numpy as np
import torch

from oracle import sp_attn_oracle as orc


def to64(x):
    return x.detach().to("cpu").to(torch.float64).numpy()


def gate(name, got, ref, dtype):
    """bf16: max-abs <= 2e-2 (scaled by ||ref||_inf / 4 once that exceeds 4, because a
    correctly rounded bf16 value of magnitude >= 8 already misses 2e-2) and relative RMS
    <= 5e-3.  fp32: relative RMS <= 1e-5 and max-abs <= 1e-5 * max(1, ||ref||_inf).
    The returned text also gives the rounding floor of the max-abs figure: the error that the
    reference itself would show after rounding to the output type."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), f"{name}: non-finite values"
    if ref.size == 0:
        return
    err = np.abs(got - ref)
    ninf = float(np.max(np.abs(ref)))
    # Relative RMS as written, against the reference's own RMS.  Only when the exact result is zero
    # (||ref||_inf < 1e-6: the dQ of a one-token group vanishes analytically) is a relative measure
    # undefined; the error is then held to the absolute gate alone.
    ref_rms = float(np.sqrt(np.mean(ref ** 2)))
    rms = float(np.sqrt(np.mean(err ** 2))) / ref_rms if ninf >= 1e-6 else 0.0
    if dtype == torch.bfloat16:
        abs_tol, rms_tol = 2e-2 * max(1.0, ninf / 4.0), 5e-3
    else:
        abs_tol, rms_tol = 1e-5 * max(1.0, ninf), 1e-5
    worst = np.unravel_index(np.argmax(err), err.shape)
    floor = ""
    if dtype == torch.bfloat16:
        rounded = torch.from_numpy(ref).to(torch.bfloat16).to(torch.float64).numpy()
        floor = f", bf16 rounding floor {float(np.max(np.abs(rounded - ref))):.3e}"
    msg = (f"{name}: max-abs {err.max():.3e} (tol {abs_tol:.3e}) at {worst}, "
           f"rel-RMS {rms:.3e} (tol {rms_tol:.1e}), ||ref||inf {ninf:.3e}{floor}")
    assert err.max() <= abs_tol and rms <= rms_tol, msg
    return msg


def gate_lse(got, ref, dtype):
    """LSE is an fp32 output on both paths; its only error sources are the fp32
    accumulation of the scores (|s| * 2^-24 * sqrt(d) at most a few 1e-6) and the fp32
    exp/log, so it is held to 1e-4 absolute (bf16 inputs) / 1e-5 relative (fp32)."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert np.all(np.isfinite(got)), "LSE: non-finite values"
    err = float(np.max(np.abs(got - ref))) if ref.size else 0.0
    tol = 1e-4 if dtype == torch.bfloat16 else 1e-5 * max(1.0, float(np.max(np.abs(ref))))
    assert err <= tol, f"LSE: max-abs {err:.3e} (tol {tol:.1e})"


def oracle_fwd(w, t):
    return orc.sp_attn_fwd_batched(t.q, t.k, t.v, w.prompt_lens(), w.Gs(), w.resp_lens_flat(),
                                   w.softmax_scale, row_block=2048)


def oracle_bwd(w, t):
    return orc.sp_attn_bwd_batched(t.q, t.k, t.v, t.d_o, w.prompt_lens(), w.Gs(), w.resp_lens_flat(),
                                   w.softmax_scale, row_block=2048)
