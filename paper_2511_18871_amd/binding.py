"""ctypes binding of libsp_attn.so.  Argument marshalling only: every step of the
attention runs in the HIP kernels behind the C ABI declared in include/sp_attn.h.
torch is used for device memory and streams, nothing else.  There is no CPU fallback:
if the library is missing, loading raises."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsp_attn.so")

SP_OK = 0
SP_ERR_INVALID_ARG, SP_ERR_UNSUPPORTED, SP_ERR_WORKSPACE, SP_ERR_DEVICE = 1, 2, 3, 4
SP_BF16, SP_F32 = 0, 1
SP_SCHED_SHARED, SP_SCHED_NAIVE_CAUSAL = 0, 1

SP_BWD_STAGE_ROWSUM, SP_BWD_STAGE_DKDV, SP_BWD_STAGE_DQ, SP_BWD_STAGE_ALL = 1, 2, 4, 7
SP_FLAG_RESPONSE_ROWS, SP_FLAG_ACCUMULATE_DKDV = 1, 2

EXPORTS = ("sp_attn_workspace_bytes", "sp_attn_reserve_bytes", "sp_attn_fwd", "sp_attn_bwd", "sp_attn_fwd_batched",
           "sp_attn_bwd_batched", "sp_attn_bwd_batched_static", "sp_attn_bwd_batched_stages", "sp_attn_fwd_multi", "sp_attn_rope", "sp_attn_rope_qk", "sp_attn_fwd_batched_ex", "sp_attn_bwd_batched_ex",
           "sp_attn_loss_workspace_bytes", "sp_attn_logprob_fwd", "sp_attn_logprob_bwd", "sp_attn_grpo_loss",
           "sp_attn_segment_table", "sp_attn_row_tile", "sp_attn_mfma_ceiling", "sp_attn_probe_atomic_add", "sp_attn_set_small_shape_steps", "sp_attn_last_error", "sp_attn_version")

_lib = None


class SpAttnError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"sp_attn status {status}: {message}")
        self.status = status


def load_library() -> ctypes.CDLL:
    """Load the in-tree library, building it first only if it has never been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from .build import build_library
        build_library(verbose=False)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
    ip = ctypes.POINTER(ctypes.c_int32)
    lib.sp_attn_workspace_bytes.restype = sz
    lib.sp_attn_workspace_bytes.argtypes = [ctypes.c_int, i64, i32, i64, i32, i32, i32, ctypes.c_int]
    lib.sp_attn_reserve_bytes.restype = sz
    lib.sp_attn_reserve_bytes.argtypes = [i64, i32, i32, ctypes.c_int]
    lib.sp_attn_fwd.restype = ctypes.c_int
    lib.sp_attn_fwd.argtypes = [vp, vp, vp, vp, vp, i32, ip, i32, i32, i32, i32, f32, ctypes.c_int, vp, sz, vp]
    lib.sp_attn_bwd.restype = ctypes.c_int
    lib.sp_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, ip, i32, i32, i32, i32, f32,
                                ctypes.c_int, vp, sz, vp]
    lib.sp_attn_fwd_batched.restype = ctypes.c_int
    lib.sp_attn_fwd_batched.argtypes = [vp, vp, vp, vp, vp, i32, ip, ip, ip, i32, i32, i32, f32, ctypes.c_int,
                                        ctypes.c_int, vp, sz, vp]
    lib.sp_attn_bwd_batched.restype = ctypes.c_int
    lib.sp_attn_bwd_batched.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, ip, ip, ip, i32, i32, i32, f32,
                                        ctypes.c_int, vp, sz, vp]
    lib.sp_attn_bwd_batched_static.restype = ctypes.c_int
    lib.sp_attn_bwd_batched_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, ip, ip, ip, i32, i32, i32, f32,
                                               ctypes.c_int, vp]
    lib.sp_attn_bwd_batched_stages.restype = ctypes.c_int
    lib.sp_attn_bwd_batched_stages.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, ip, ip, ip, i32, i32, i32,
                                               f32, ctypes.c_int, ctypes.c_uint32, vp, sz, vp]
    pp = ctypes.POINTER(ctypes.c_void_p)
    lib.sp_attn_fwd_multi.restype = ctypes.c_int
    lib.sp_attn_fwd_multi.argtypes = [i32, pp, pp, pp, pp, pp, i32, ip, ip, ip, i32, i32, i32, f32, ctypes.c_int, vp, sz, vp]
    lib.sp_attn_fwd_batched_ex.restype = ctypes.c_int
    lib.sp_attn_fwd_batched_ex.argtypes = [vp, vp, vp, vp, vp, i32, ip, ip, ip, i32, i32, i32, f32, ctypes.c_int,
                                           ctypes.c_int, ctypes.c_uint32, vp, vp, sz, vp]
    lib.sp_attn_bwd_batched_ex.restype = ctypes.c_int
    lib.sp_attn_bwd_batched_ex.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, ip, ip, ip, i32, i32, i32, f32,
                                           ctypes.c_int, ctypes.c_uint32, ctypes.c_uint32, vp, vp, sz, vp]
    i64 = ctypes.c_int64
    lib.sp_attn_loss_workspace_bytes.restype = sz
    lib.sp_attn_loss_workspace_bytes.argtypes = [i64, i32, i64]
    lib.sp_attn_logprob_fwd.restype = ctypes.c_int
    lib.sp_attn_logprob_fwd.argtypes = [vp, vp, vp, vp, i64, i32, ip, ip, ip, ctypes.c_int, vp, sz, vp]
    lib.sp_attn_logprob_bwd.restype = ctypes.c_int
    lib.sp_attn_logprob_bwd.argtypes = [vp, vp, vp, vp, vp, i64, i32, ip, ip, ip, ctypes.c_int, vp, sz, vp]
    lib.sp_attn_grpo_loss.restype = ctypes.c_int
    lib.sp_attn_grpo_loss.argtypes = [vp, vp, vp, vp, f32, f32, f32, vp, vp, i32, ip, ip, ip, vp, sz, vp]
    lib.sp_attn_rope.restype = ctypes.c_int
    lib.sp_attn_rope.argtypes = [vp, vp, i32, i32, i32, ip, ip, ip, i32, ctypes.c_double, ctypes.c_int, vp, sz, vp]
    lib.sp_attn_rope_qk.restype = ctypes.c_int
    lib.sp_attn_rope_qk.argtypes = [vp, vp, i32, vp, vp, i32, i32, i32, ip, ip, ip, i32, ctypes.c_double, ctypes.c_int, vp, sz, vp]
    lib.sp_attn_segment_table.restype = ctypes.c_int
    lib.sp_attn_segment_table.argtypes = [i32, ip, ip, ip, ip, sz, ctypes.POINTER(sz)]
    lib.sp_attn_row_tile.restype = ctypes.c_int
    lib.sp_attn_row_tile.argtypes = [i32, ip, ip, ip, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64),
                                     ctypes.POINTER(ctypes.c_int64)]
    lib.sp_attn_mfma_ceiling.restype = ctypes.c_int
    lib.sp_attn_mfma_ceiling.argtypes = [i32, vp, vp, i32, i32, vp, vp]
    lib.sp_attn_probe_atomic_add.restype = ctypes.c_int
    lib.sp_attn_probe_atomic_add.argtypes = [vp, i64, i32, i32, i32, i32, vp]
    lib.sp_attn_set_small_shape_steps.restype = None
    lib.sp_attn_set_small_shape_steps.argtypes = [i32]
    lib.sp_attn_last_error.restype = ctypes.c_char_p
    lib.sp_attn_last_error.argtypes = []
    lib.sp_attn_version.restype = ctypes.c_char_p
    lib.sp_attn_version.argtypes = []
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != SP_OK:
        raise SpAttnError(status, load_library().sp_attn_last_error().decode())


def sp_attn_segment_table(prompt_lens: Sequence[int], Gs: Sequence[int], resp_lens_flat: Sequence[int]) -> list:
    """The segment table (list of ints) that a call with these host arrays hands to its kernels."""
    lib = load_library()
    n = ctypes.c_size_t(0)
    args = (len(prompt_lens), _i32(prompt_lens), _i32(Gs), _i32(resp_lens_flat))
    st = lib.sp_attn_segment_table(*args, None, 0, ctypes.byref(n))
    if st != SP_ERR_WORKSPACE:
        _check(st)
    buf = (ctypes.c_int32 * n.value)()
    _check(lib.sp_attn_segment_table(*args, buf, n.value, ctypes.byref(n)))
    return list(buf)


def sp_attn_row_tile(prompt_lens: Sequence[int], Gs: Sequence[int], resp_lens_flat: Sequence[int]):
    """(rows, steps_256, steps_128): the workgroup shape (256 or 128 query rows) that a bf16 call on this packing
    takes, and the 64-key steps per q head of either tiling.  Host arithmetic only."""
    lib = load_library()
    rows = ctypes.c_int32(0)
    s256, s128 = ctypes.c_int64(0), ctypes.c_int64(0)
    _check(lib.sp_attn_row_tile(len(prompt_lens), _i32(prompt_lens), _i32(Gs), _i32(resp_lens_flat),
                                ctypes.byref(rows), ctypes.byref(s256), ctypes.byref(s128)))
    return rows.value, s256.value, s128.value


def _i32(xs: Sequence[int]):
    arr = (ctypes.c_int32 * max(1, len(xs)))(*xs)
    return arr


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return SP_BF16
    if t.dtype == torch.float32:
        return SP_F32
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def workspace_bytes(is_bwd: bool, total_tokens: int, n_groups: int, total_responses: int, n_q_heads: int,
                    n_kv_heads: int, head_dim: int, dtype_code: int) -> int:
    return load_library().sp_attn_workspace_bytes(int(is_bwd), total_tokens, n_groups, total_responses, n_q_heads,
                                                  n_kv_heads, head_dim, dtype_code)


def reserve_bytes(total_tokens: int, n_q_heads: int, head_dim: int, dtype_code: int) -> int:
    return load_library().sp_attn_reserve_bytes(total_tokens, n_q_heads, head_dim, dtype_code)


def _workspace(is_bwd, q, n_groups, n_resp, n_kv_heads, workspace, o=None, reserve=False):
    """The workspace tensor of a call.  When the caller passes none: a forward allocates one that also has
    room for the forward-to-backward reserve and hangs it on the output tensor it returns (attribute
    ``_sp_workspace``); the backward that is given that output finds it there and passes it on, which is
    all the library needs to use the reserve.  Plumbing only: what the reserve is and whether it is valid
    is decided by the library."""
    T, Hq, d = q.shape
    if workspace is not None:
        return workspace
    if is_bwd and o is not None and getattr(o, "_sp_workspace", None) is not None:
        return o._sp_workspace
    need = workspace_bytes(is_bwd or reserve, T, n_groups, n_resp, Hq, n_kv_heads, d, _dtype_code(q))
    if reserve:
        need += reserve_bytes(T, Hq, d, _dtype_code(q))
    workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    if reserve and o is not None:
        o._sp_workspace = workspace        # sized for the backward too
    return workspace


def sp_attn_fwd(q, k, v, prompt_len: int, resp_lens: Sequence[int], softmax_scale: float,
                o=None, lse=None, workspace=None, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Forward for one group.  q [T,Hq,d]; k, v [T,Hkv,d] on the GPU.  Returns (o, lse)."""
    lib = load_library()
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    o = torch.empty_like(q) if o is None else o
    lse = torch.empty(Hq, T, dtype=torch.float32, device=q.device) if lse is None else lse
    workspace = _workspace(False, q, 1, len(resp_lens), Hkv, workspace, o=o, reserve=True)
    _check(lib.sp_attn_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(), prompt_len,
                           _i32(resp_lens), len(resp_lens), Hq, Hkv, d, softmax_scale, _dtype_code(q),
                           workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return o, lse


def sp_attn_bwd(q, k, v, o, lse, d_o, prompt_len: int, resp_lens: Sequence[int], softmax_scale: float,
                dq=None, dk=None, dv=None, workspace=None, stream=None):
    """Backward for one group.  Returns (dq, dk, dv)."""
    lib = load_library()
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(k) if dk is None else dk
    dv = torch.empty_like(v) if dv is None else dv
    workspace = _workspace(True, q, 1, len(resp_lens), Hkv, workspace, o=o)
    _check(lib.sp_attn_bwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(), d_o.data_ptr(),
                           dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), prompt_len, _i32(resp_lens),
                           len(resp_lens), Hq, Hkv, d, softmax_scale, _dtype_code(q), workspace.data_ptr(),
                           workspace.numel(), _stream_ptr(stream)))
    return dq, dk, dv


def sp_attn_fwd_batched(q, k, v, prompt_lens: Sequence[int], Gs: Sequence[int], resp_lens_flat: Sequence[int],
                        softmax_scale: float, schedule: int = SP_SCHED_SHARED, o=None, lse=None, workspace=None,
                        stream=None):
    lib = load_library()
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    o = torch.empty_like(q) if o is None else o
    lse = torch.empty(Hq, T, dtype=torch.float32, device=q.device) if lse is None else lse
    workspace = _workspace(False, q, len(prompt_lens), len(resp_lens_flat), Hkv, workspace, o=o, reserve=True)
    _check(lib.sp_attn_fwd_batched(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(),
                                   len(prompt_lens), _i32(prompt_lens), _i32(Gs), _i32(resp_lens_flat), Hq, Hkv, d,
                                   softmax_scale, _dtype_code(q), schedule, workspace.data_ptr(),
                                   workspace.numel(), _stream_ptr(stream)))
    return o, lse


def sp_attn_fwd_multi(qs, ks, vs, prompt_lens: Sequence[int], Gs: Sequence[int], resp_lens_flat: Sequence[int],
                      softmax_scale: float, os=None, lses=None, workspace=None, stream=None):
    """Forward of several (q, k, v) sets that share one packing, in one launch.  Returns (os, lses)."""
    lib = load_library()
    n = len(qs)
    T, Hq, d = qs[0].shape
    Hkv = ks[0].shape[1]
    os = [torch.empty_like(q) for q in qs] if os is None else os
    lses = [torch.empty(Hq, T, dtype=torch.float32, device=qs[0].device) for _ in qs] if lses is None else lses
    workspace = _workspace(False, qs[0], len(prompt_lens), len(resp_lens_flat), Hkv, workspace)
    arr = lambda ts: (ctypes.c_void_p * max(1, len(ts)))(*[t.data_ptr() for t in ts])
    _check(lib.sp_attn_fwd_multi(n, arr(qs), arr(ks), arr(vs), arr(os), arr(lses), len(prompt_lens),
                                 _i32(prompt_lens), _i32(Gs), _i32(resp_lens_flat), Hq, Hkv, d, softmax_scale,
                                 _dtype_code(qs[0]), workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return os, lses


def sp_attn_fwd_batched_ex(q, k, v, prompt_lens: Sequence[int], Gs: Sequence[int], resp_lens_flat: Sequence[int],
                           softmax_scale: float, flags: int, o=None, lse=None, workspace=None, stream=None,
                           schedule: int = SP_SCHED_SHARED, o_lo=None):
    """sp_attn_fwd_batched with a flags word (SP_FLAG_RESPONSE_ROWS).  Rows that the flags exclude keep
    whatever ``o`` / ``lse`` held."""
    lib = load_library()
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    o = torch.empty_like(q) if o is None else o
    lse = torch.empty(Hq, T, dtype=torch.float32, device=q.device) if lse is None else lse
    workspace = _workspace(False, q, len(prompt_lens), len(resp_lens_flat), Hkv, workspace, o=o, reserve=o_lo is None)
    _check(lib.sp_attn_fwd_batched_ex(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(),
                                      len(prompt_lens), _i32(prompt_lens), _i32(Gs), _i32(resp_lens_flat), Hq, Hkv, d,
                                      softmax_scale, _dtype_code(q), schedule, flags,
                                      None if o_lo is None else o_lo.data_ptr(), workspace.data_ptr(),
                                      workspace.numel(), _stream_ptr(stream)))
    return o, lse


def sp_attn_bwd_batched_ex(q, k, v, o, lse, d_o, prompt_lens: Sequence[int], Gs: Sequence[int],
                           resp_lens_flat: Sequence[int], softmax_scale: float, flags: int, dq=None, dk=None, dv=None,
                           workspace=None, stream=None, stages: int = 7, o_lo=None):
    """sp_attn_bwd_batched with a flags word (SP_FLAG_RESPONSE_ROWS, SP_FLAG_ACCUMULATE_DKDV)."""
    lib = load_library()
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(k) if dk is None else dk
    dv = torch.empty_like(v) if dv is None else dv
    workspace = _workspace(True, q, len(prompt_lens), len(resp_lens_flat), Hkv, workspace, o=o)
    _check(lib.sp_attn_bwd_batched_ex(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(),
                                      d_o.data_ptr(), dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), len(prompt_lens),
                                      _i32(prompt_lens), _i32(Gs), _i32(resp_lens_flat), Hq, Hkv, d, softmax_scale,
                                      _dtype_code(q), stages, flags, None if o_lo is None else o_lo.data_ptr(),
                                      workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return dq, dk, dv


def _loss_ws(T, n_groups, n_resp, device, workspace):
    if workspace is None:
        need = load_library().sp_attn_loss_workspace_bytes(T, n_groups, n_resp)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
    return workspace


def sp_attn_logprob_fwd(logits, labels, prompt_lens: Sequence[int], Gs: Sequence[int], resp_lens_flat: Sequence[int],
                        logp=None, lse=None, workspace=None, stream=None):
    """Log-probability of labels[t] at every response row t of logits [T, V].  Returns (logp, lse);
    prompt rows keep whatever the output tensors held (zeros when allocated here)."""
    lib = load_library()
    T, V = logits.shape
    logp = torch.zeros(T, dtype=torch.float32, device=logits.device) if logp is None else logp
    lse = torch.zeros(T, dtype=torch.float32, device=logits.device) if lse is None else lse
    workspace = _loss_ws(T, len(prompt_lens), len(resp_lens_flat), logits.device, workspace)
    _check(lib.sp_attn_logprob_fwd(logits.data_ptr(), labels.data_ptr(), logp.data_ptr(), lse.data_ptr(), V,
                                   len(prompt_lens), _i32(prompt_lens), _i32(Gs), _i32(resp_lens_flat),
                                   _dtype_code(logits), workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return logp, lse


def sp_attn_logprob_bwd(logits, labels, lse, g, prompt_lens: Sequence[int], Gs: Sequence[int],
                        resp_lens_flat: Sequence[int], dlogits=None, workspace=None, stream=None):
    lib = load_library()
    T, V = logits.shape
    dlogits = torch.zeros_like(logits) if dlogits is None else dlogits
    workspace = _loss_ws(T, len(prompt_lens), len(resp_lens_flat), logits.device, workspace)
    _check(lib.sp_attn_logprob_bwd(logits.data_ptr(), labels.data_ptr(), lse.data_ptr(), g.data_ptr(),
                                   dlogits.data_ptr(), V, len(prompt_lens), _i32(prompt_lens), _i32(Gs),
                                   _i32(resp_lens_flat), _dtype_code(logits), workspace.data_ptr(), workspace.numel(),
                                   _stream_ptr(stream)))
    return dlogits


def sp_attn_grpo_loss(logp, logp_old, logp_ref, adv, prompt_lens: Sequence[int], Gs: Sequence[int],
                      resp_lens_flat: Sequence[int], eps_low: float = 0.2, eps_high: float = 0.2, beta: float = 0.02,
                      g=None, workspace=None, stream=None):
    """GRPO objective over the response rows.  Returns (loss [1], g [T] = dloss/dlogp)."""
    lib = load_library()
    T = logp.shape[0]
    loss = torch.zeros(1, dtype=torch.float32, device=logp.device)
    g = torch.zeros(T, dtype=torch.float32, device=logp.device) if g is None else g
    workspace = _loss_ws(T, len(prompt_lens), len(resp_lens_flat), logp.device, workspace)
    _check(lib.sp_attn_grpo_loss(logp.data_ptr(), logp_old.data_ptr(), logp_ref.data_ptr(), adv.data_ptr(), eps_low,
                                 eps_high, beta, loss.data_ptr(), g.data_ptr(), len(prompt_lens), _i32(prompt_lens),
                                 _i32(Gs), _i32(resp_lens_flat), workspace.data_ptr(), workspace.numel(),
                                 _stream_ptr(stream)))
    return loss, g


def sp_attn_rope(x, prompt_lens: Sequence[int], Gs: Sequence[int], resp_lens_flat: Sequence[int], rope_base: float,
                 inverse: bool = False, out=None, workspace=None, stream=None):
    """Rotary embedding of x [T, H, d] at the restarted position indices; returns the rotated tensor
    (``out`` may be x itself)."""
    lib = load_library()
    T, H, d = x.shape
    out = torch.empty_like(x) if out is None else out
    if workspace is None:
        need = workspace_bytes(False, T, len(prompt_lens), len(resp_lens_flat), H, H, d, _dtype_code(x))
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    _check(lib.sp_attn_rope(x.data_ptr(), out.data_ptr(), H, int(inverse), len(prompt_lens), _i32(prompt_lens),
                            _i32(Gs), _i32(resp_lens_flat), d, float(rope_base), _dtype_code(x),
                            workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return out


def sp_attn_rope_qk(q, k, prompt_lens: Sequence[int], Gs: Sequence[int], resp_lens_flat: Sequence[int], rope_base: float,
                    inverse: bool = False, q_out=None, k_out=None, workspace=None, stream=None):
    """Rotary embedding of q [T, Hq, d] and k [T, Hkv, d] in one launch; returns (q_out, k_out)."""
    lib = load_library()
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    q_out = torch.empty_like(q) if q_out is None else q_out
    k_out = torch.empty_like(k) if k_out is None else k_out
    if workspace is None:
        need = workspace_bytes(False, T, len(prompt_lens), len(resp_lens_flat), Hq, Hq, d, _dtype_code(q))
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    _check(lib.sp_attn_rope_qk(q.data_ptr(), q_out.data_ptr(), Hq, k.data_ptr(), k_out.data_ptr(), Hkv, int(inverse),
                               len(prompt_lens), _i32(prompt_lens), _i32(Gs), _i32(resp_lens_flat), d, float(rope_base),
                               _dtype_code(q), workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return q_out, k_out


def sp_attn_bwd_batched(q, k, v, o, lse, d_o, prompt_lens: Sequence[int], Gs: Sequence[int],
                        resp_lens_flat: Sequence[int], softmax_scale: float, dq=None, dk=None, dv=None,
                        workspace=None, stream=None):
    lib = load_library()
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(k) if dk is None else dk
    dv = torch.empty_like(v) if dv is None else dv
    workspace = _workspace(True, q, len(prompt_lens), len(resp_lens_flat), Hkv, workspace, o=o)
    _check(lib.sp_attn_bwd_batched(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(),
                                   d_o.data_ptr(), dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), len(prompt_lens),
                                   _i32(prompt_lens), _i32(Gs), _i32(resp_lens_flat), Hq, Hkv, d, softmax_scale,
                                   _dtype_code(q), workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return dq, dk, dv


def sp_attn_probe_atomic_add(buf, rows: int, heads: int, steps: int, n_blocks: int = 512, layout: int = 0, stream=None) -> int:
    """Enqueue the atomic-add measurement loop; returns the bytes the launch adds."""
    st = load_library().sp_attn_probe_atomic_add(buf.data_ptr(), rows, heads, steps, n_blocks, layout, _stream_ptr(stream))
    if st != SP_OK:
        raise SpAttnError(st, "sp_attn_probe_atomic_add: invalid argument or launch failure")
    return n_blocks * steps * 32768


def set_small_shape_steps(steps: int) -> None:
    """Threshold (mean 64-key steps per 256-row workgroup) below which calls take the 128-row kernel shape."""
    load_library().sp_attn_set_small_shape_steps(steps)


def sp_attn_mfma_ceiling(lds_operands: int, a, b, iters: int, out, n_blocks: int = 256, stream=None) -> float:
    """Enqueue the MFMA-only measurement loop; returns the FLOPs the launch executes."""
    lib = load_library()
    st = lib.sp_attn_mfma_ceiling(lds_operands, a.data_ptr(), b.data_ptr(), iters, n_blocks, out.data_ptr(),
                                  _stream_ptr(stream))
    if st != SP_OK:
        raise SpAttnError(st, "sp_attn_mfma_ceiling: invalid argument or launch failure")
    return float(n_blocks) * 8 * iters * 16 * 32768.0


def sp_attn_bwd_batched_static(q, k, v, o, lse, d_o, dq, dk, dv, prompt_lens: Sequence[int], Gs: Sequence[int],
                               resp_lens_flat: Sequence[int], softmax_scale: float, stream=None) -> None:
    """sp_attn_bwd_batched on the library's built-in device scratch: no workspace, and nothing is
    allocated (the caller passes every output)."""
    lib = load_library()
    T, Hq, d = q.shape
    _check(lib.sp_attn_bwd_batched_static(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(),
                                          d_o.data_ptr(), dq.data_ptr(), dk.data_ptr(), dv.data_ptr(),
                                          len(prompt_lens), _i32(prompt_lens), _i32(Gs), _i32(resp_lens_flat), Hq,
                                          k.shape[1], d, softmax_scale, _dtype_code(q), _stream_ptr(stream)))


def sp_attn_bwd_batched_stages(q, k, v, o, lse, d_o, prompt_lens: Sequence[int], Gs: Sequence[int],
                               resp_lens_flat: Sequence[int], softmax_scale: float, stages: int, workspace,
                               dq=None, dk=None, dv=None, stream=None) -> None:
    """Enqueue a subset of the backward stages (SP_BWD_STAGE_* bits).  The caller passes the
    workspace, because D written by the ROWSUM stage is read by the other two."""
    lib = load_library()
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    ptr = lambda x: None if x is None else x.data_ptr()
    _check(lib.sp_attn_bwd_batched_stages(q.data_ptr(), k.data_ptr(), v.data_ptr(), ptr(o), lse.data_ptr(),
                                          d_o.data_ptr(), ptr(dq), ptr(dk), ptr(dv), len(prompt_lens),
                                          _i32(prompt_lens), _i32(Gs), _i32(resp_lens_flat), Hq, Hkv, d,
                                          softmax_scale, _dtype_code(q), stages, workspace.data_ptr(),
                                          workspace.numel(), _stream_ptr(stream)))
