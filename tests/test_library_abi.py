"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header
declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2511_18871_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return B.load_library()


def declared_symbols():
    with open(os.path.join(ROOT, "include", "sp_attn.h")) as f:
        text = re.sub(r"/\*.*?\*/", "", f.read(), flags=re.S)
    return sorted(set(re.findall(r"\b(sp_attn_\w+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = declared_symbols()
    assert set(names) == set(B.EXPORTS)
    raw = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert getattr(raw, n) is not None


def test_version_and_workspace_size(lib):
    assert lib.sp_attn_version().decode() == "0.1"
    fwd = B.workspace_bytes(False, 1000, 2, 7, 8, 2, 128, B.SP_BF16)
    bwd = B.workspace_bytes(True, 1000, 2, 7, 8, 2, 128, B.SP_BF16)
    assert fwd >= (4 + 6 * 2 + 7 + 2) * 4 and fwd % 256 == 0
    assert bwd - fwd >= 8 * 1000 * 4
    assert B.workspace_bytes(False, 0, 1, 0, 8, 2, 128, B.SP_BF16) == 0


def _call_fwd(lib, *, q=0x1000, k=0x1000, v=0x1000, o=0x1000, lse=0x1000, lp=4, lens=(3,), Hq=4, Hkv=2, d=128,
              scale=0.1, dtype=B.SP_BF16, ws=0x1000, ws_bytes=1 << 20):
    arr = (ctypes.c_int32 * max(1, len(lens)))(*lens)
    return lib.sp_attn_fwd(q, k, v, o, lse, lp, arr, len(lens), Hq, Hkv, d, scale, dtype, ws, ws_bytes, None)


def test_invalid_arguments_are_rejected_on_the_host(lib):
    """Every call below must fail validation, so no kernel is launched and the fake
    device addresses are never dereferenced."""
    assert _call_fwd(lib, q=None) == B.SP_ERR_INVALID_ARG
    assert _call_fwd(lib, q=0x1004) == B.SP_ERR_INVALID_ARG
    assert _call_fwd(lib, lp=-1) == B.SP_ERR_INVALID_ARG
    assert _call_fwd(lib, lens=(3, -2)) == B.SP_ERR_INVALID_ARG
    assert _call_fwd(lib, lp=0, lens=(0, 0)) == B.SP_ERR_INVALID_ARG      # empty group
    assert _call_fwd(lib, Hq=5, Hkv=2) == B.SP_ERR_INVALID_ARG
    assert _call_fwd(lib, scale=0.0) == B.SP_ERR_INVALID_ARG
    assert _call_fwd(lib, scale=float("nan")) == B.SP_ERR_INVALID_ARG
    assert _call_fwd(lib, d=96) == B.SP_ERR_UNSUPPORTED
    assert _call_fwd(lib, d=64) == B.SP_ERR_UNSUPPORTED                   # bf16 needs 128
    assert _call_fwd(lib, dtype=7) == B.SP_ERR_UNSUPPORTED
    assert _call_fwd(lib, ws=None) == B.SP_ERR_WORKSPACE
    assert _call_fwd(lib, ws_bytes=16) == B.SP_ERR_WORKSPACE
    assert b"workspace" in lib.sp_attn_last_error()


def test_bad_stage_mask_is_rejected(lib):
    one = (ctypes.c_int32 * 1)(4)
    g = (ctypes.c_int32 * 1)(1)
    r = (ctypes.c_int32 * 1)(3)
    for stages in (0, 8, 15):
        st = lib.sp_attn_bwd_batched_stages(0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000,
                                            1, one, g, r, 4, 2, 128, 0.1, B.SP_BF16, stages, 0x1000, 1 << 20, None)
        assert st == B.SP_ERR_INVALID_ARG


def test_multi_set_forward_rejects_bad_set_counts_and_arrays(lib):
    one = (ctypes.c_int32 * 1)(4)
    g = (ctypes.c_int32 * 1)(1)
    r = (ctypes.c_int32 * 1)(3)
    ptrs = (ctypes.c_void_p * 5)(*([0x1000] * 5))
    def call(n, q=ptrs, ws=0x1000):
        return lib.sp_attn_fwd_multi(n, q, ptrs, ptrs, ptrs, ptrs, 1, one, g, r, 4, 2, 128, 0.1, B.SP_BF16, ws,
                                     1 << 20, None)
    assert call(0) == B.SP_ERR_INVALID_ARG
    assert call(5) == B.SP_ERR_INVALID_ARG
    assert call(2, q=None) == B.SP_ERR_INVALID_ARG
    bad = (ctypes.c_void_p * 5)(0x1000, 0x1008, 0x1000, 0x1000, 0x1000)
    assert call(2, q=bad) == B.SP_ERR_INVALID_ARG           # set 1: misaligned q
    assert call(3, ws=None) == B.SP_ERR_WORKSPACE


def test_rope_rejects_bad_arguments(lib):
    one = (ctypes.c_int32 * 1)(4)
    g = (ctypes.c_int32 * 1)(1)
    r = (ctypes.c_int32 * 1)(3)
    def call(x=0x1000, y=0x1000, H=2, d=128, base=10000.0, dtype=B.SP_BF16, ws=0x1000):
        return lib.sp_attn_rope(x, y, H, 0, 1, one, g, r, d, base, dtype, ws, 1 << 20, None)
    assert call(x=None) == B.SP_ERR_INVALID_ARG
    assert call(y=0x1002) == B.SP_ERR_INVALID_ARG
    assert call(H=0) == B.SP_ERR_INVALID_ARG
    assert call(base=1.0) == B.SP_ERR_INVALID_ARG
    assert call(base=float("inf")) == B.SP_ERR_INVALID_ARG
    assert call(d=96) == B.SP_ERR_UNSUPPORTED
    assert call(dtype=5) == B.SP_ERR_UNSUPPORTED
    assert call(ws=None) == B.SP_ERR_WORKSPACE


def test_flags_word_is_validated(lib):
    one = (ctypes.c_int32 * 1)(4)
    g = (ctypes.c_int32 * 1)(1)
    r = (ctypes.c_int32 * 1)(3)
    P = 0x1000
    def fwd(flags):
        return lib.sp_attn_fwd_batched_ex(P, P, P, P, P, 1, one, g, r, 4, 2, 128, 0.1, B.SP_BF16, B.SP_SCHED_SHARED,
                                          flags, None, None, 0, None)
    def bwd(flags):
        return lib.sp_attn_bwd_batched_ex(P, P, P, P, P, P, P, P, P, 1, one, g, r, 4, 2, 128, 0.1, B.SP_BF16, 7, flags,
                                          None, None, 0, None)
    assert fwd(4) == B.SP_ERR_INVALID_ARG and bwd(8) == B.SP_ERR_INVALID_ARG
    assert fwd(B.SP_FLAG_ACCUMULATE_DKDV) == B.SP_ERR_INVALID_ARG
    # valid flags pass the flag check and fail later, at the (missing) workspace
    assert fwd(B.SP_FLAG_RESPONSE_ROWS) == B.SP_ERR_WORKSPACE
    assert bwd(B.SP_FLAG_RESPONSE_ROWS | B.SP_FLAG_ACCUMULATE_DKDV) == B.SP_ERR_WORKSPACE
    # the optional residual tensor: alignment, and bf16 only
    assert lib.sp_attn_fwd_batched_ex(P, P, P, P, P, 1, one, g, r, 4, 2, 128, 0.1, B.SP_BF16, B.SP_SCHED_SHARED, 0,
                                      0x1008, P, 1 << 20, None) == B.SP_ERR_INVALID_ARG
    assert lib.sp_attn_fwd_batched_ex(P, P, P, P, P, 1, one, g, r, 4, 2, 64, 0.1, B.SP_F32, B.SP_SCHED_SHARED, 0,
                                      P, P, 1 << 20, None) == B.SP_ERR_UNSUPPORTED


def test_loss_calls_reject_bad_arguments(lib):
    one = (ctypes.c_int32 * 1)(4)
    g = (ctypes.c_int32 * 1)(1)
    r = (ctypes.c_int32 * 1)(3)
    P = 0x1000
    assert lib.sp_attn_loss_workspace_bytes(7, 1, 1) >= (4 + 6 + 1 + 1) * 4 + 8
    assert lib.sp_attn_loss_workspace_bytes(0, 1, 1) == 0
    f = lambda **kw: lib.sp_attn_logprob_fwd(kw.get("z", P), P, P, P, kw.get("V", 100), 1, one, g, r,
                                             kw.get("dtype", B.SP_BF16), kw.get("ws", P), 1 << 20, None)
    assert f(z=None) == B.SP_ERR_INVALID_ARG and f(z=0x1002) == B.SP_ERR_INVALID_ARG
    assert f(V=0) == B.SP_ERR_INVALID_ARG
    assert f(dtype=9) == B.SP_ERR_UNSUPPORTED
    assert f(ws=None) == B.SP_ERR_WORKSPACE
    b = lambda **kw: lib.sp_attn_logprob_bwd(P, P, P, P, kw.get("dz", P), 100, 1, one, g, r, B.SP_F32, kw.get("ws", P),
                                             1 << 20, None)
    assert b(dz=None) == B.SP_ERR_INVALID_ARG and b(ws=None) == B.SP_ERR_WORKSPACE
    q = lambda **kw: lib.sp_attn_grpo_loss(P, P, P, kw.get("adv", P), kw.get("el", 0.2), kw.get("eh", 0.2),
                                           kw.get("beta", 0.02), P, P, 1, one, g, r, kw.get("ws", P), 1 << 20, None)
    assert q(adv=None) == B.SP_ERR_INVALID_ARG
    assert q(el=1.0) == B.SP_ERR_INVALID_ARG and q(el=-0.1) == B.SP_ERR_INVALID_ARG
    assert q(eh=float("inf")) == B.SP_ERR_INVALID_ARG and q(beta=float("nan")) == B.SP_ERR_INVALID_ARG
    assert q(ws=None) == B.SP_ERR_WORKSPACE


def test_segment_table_contents(lib):
    """The host logic that turns (prompt_lens, Gs, resp_lens) into the table the kernels read: token
    bases, per-group offsets and the running tile counts that the tile -> group bisection relies on."""
    import numpy as np
    rng = np.random.default_rng(5)
    for trial in range(40):
        ng = int(rng.integers(1, 30))
        pl = [int(x) for x in rng.integers(0, 700, ng)]
        Gs = [int(x) for x in rng.integers(0, 6, ng)]
        rl = [int(x) for g in Gs for x in rng.integers(0, 300, g)]
        if trial == 0:
            pl, Gs, rl = [0, 5], [2, 0], [0, 256]          # a zero-length response, a group with no response
        for g in range(ng if trial else 2):                # every group needs at least one token
            if pl[g] + sum(rl[sum(Gs[:g]):sum(Gs[:g + 1])]) == 0:
                pl[g] = 1
        ng = len(pl)
        tab = B.sp_attn_segment_table(pl, Gs, rl)
        totals = [pl[g] + sum(rl[sum(Gs[:g]):sum(Gs[:g + 1])]) for g in range(ng)]
        assert tab[0] == ng and tab[1] == sum(totals) and tab[2] == len(tab) == 4 + 8 * ng + sum(Gs) + ng and tab[3] == 0
        next_off, tok, t256, t128, r = 4 + 8 * ng, 0, 0, 0, 0
        for g in range(ng):
            e = tab[4 + 8 * g: 12 + 8 * g]
            assert e == [tok, pl[g], totals[g], next_off, Gs[g], t256, t128, 0], (trial, g, e)
            offs = tab[next_off: next_off + Gs[g] + 1]
            want = [pl[g]]
            for i in range(Gs[g]):
                want.append(want[-1] + rl[r + i])
            assert offs == want and offs[-1] == totals[g]
            r += Gs[g]
            next_off += Gs[g] + 1
            tok += totals[g]
            t256 += -(-totals[g] // 256)
            t128 += -(-totals[g] // 128)
        assert next_off == len(tab)


def test_segment_table_errors(lib):
    n = ctypes.c_size_t(0)
    i32 = lambda xs: (ctypes.c_int32 * max(1, len(xs)))(*xs)
    buf = (ctypes.c_int32 * 4)()
    # too small a buffer: the needed size is still reported
    assert lib.sp_attn_segment_table(1, i32([10]), i32([2]), i32([3, 4]), buf, 4, ctypes.byref(n)) == B.SP_ERR_WORKSPACE
    assert n.value == 4 + 8 + 3
    assert lib.sp_attn_segment_table(1, i32([10]), i32([2]), i32([3, -4]), None, 0, ctypes.byref(n)) == B.SP_ERR_INVALID_ARG
    assert lib.sp_attn_segment_table(1, i32([0]), i32([1]), i32([0]), None, 0, ctypes.byref(n)) == B.SP_ERR_INVALID_ARG
    assert b"empty" in lib.sp_attn_last_error()
    assert lib.sp_attn_segment_table(0, i32([]), i32([]), i32([]), None, 0, ctypes.byref(n)) == B.SP_ERR_INVALID_ARG
    assert lib.sp_attn_segment_table(1, i32([10]), i32([0]), None, None, 0, None) == B.SP_ERR_INVALID_ARG


def test_reserve_and_workspace_sizes(lib):
    """The forward-to-backward reserve: size formula, zero for fp32 and for arguments no call accepts; a
    workspace with room for it is the backward's size plus the reserve."""
    T, Hq, d = 1000, 8, 128
    assert B.reserve_bytes(T, Hq, d, B.SP_BF16) == (T * Hq * d * 2 + 255) // 256 * 256
    assert B.reserve_bytes(T, Hq, d, B.SP_F32) == 0
    assert B.reserve_bytes(0, Hq, d, B.SP_BF16) == 0 and B.reserve_bytes(T, 0, d, B.SP_BF16) == 0
    fwd = B.workspace_bytes(False, T, 3, 9, Hq, 2, d, B.SP_BF16)
    bwd = B.workspace_bytes(True, T, 3, 9, Hq, 2, d, B.SP_BF16)
    # tag block, table, schedule (two ints per token and a descriptor per tile of 256 and of 128)
    assert fwd >= 256 + (4 + 8 * 3 + 9 + 3) * 4 + 8 * T + 32 * (T // 256 + T // 128)
    assert bwd > fwd and fwd % 256 == 0 and bwd % 256 == 0
    # more groups or more responses never need less
    assert B.workspace_bytes(True, T, 30, 90, Hq, 2, d, B.SP_BF16) >= bwd


def test_measurement_aids_and_knob_reject_bad_arguments(lib):
    P = 0x1000
    assert lib.sp_attn_mfma_ceiling(3, P, P, 10, 256, P, None) == B.SP_ERR_INVALID_ARG
    assert lib.sp_attn_mfma_ceiling(0, None, P, 10, 256, P, None) == B.SP_ERR_INVALID_ARG
    assert lib.sp_attn_mfma_ceiling(0, 0x1004, P, 10, 256, P, None) == B.SP_ERR_INVALID_ARG
    assert lib.sp_attn_mfma_ceiling(0, P, P, 0, 256, P, None) == B.SP_ERR_INVALID_ARG
    assert lib.sp_attn_probe_atomic_add(None, 64, 8, 1, 1, 0, None) == B.SP_ERR_INVALID_ARG
    assert lib.sp_attn_probe_atomic_add(P, 63, 8, 1, 1, 0, None) == B.SP_ERR_INVALID_ARG
    assert lib.sp_attn_probe_atomic_add(P, 64, 8, 1, 1, 2, None) == B.SP_ERR_INVALID_ARG
    B.set_small_shape_steps(0)
    B.set_small_shape_steps(-1)            # back to the default; no return value, must not raise


def test_rope_qk_argument_checks(lib):
    i32 = lambda xs: (ctypes.c_int32 * max(1, len(xs)))(*xs)
    P = 0x1000
    f = lambda **kw: lib.sp_attn_rope_qk(kw.get("q", P), P, kw.get("Hq", 4), kw.get("k", P), kw.get("ko", P), 2, 0, 1,
                                         i32([10]), i32([1]), i32([5]), kw.get("d", 128), kw.get("base", 1e4), B.SP_BF16,
                                         kw.get("ws", P), 1 << 20, None)
    assert f(q=None) == B.SP_ERR_INVALID_ARG and f(k=None) == B.SP_ERR_INVALID_ARG and f(ko=None) == B.SP_ERR_INVALID_ARG
    assert f(k=0x1008) == B.SP_ERR_INVALID_ARG
    assert f(Hq=0) == B.SP_ERR_INVALID_ARG and f(base=1.0) == B.SP_ERR_INVALID_ARG
    assert f(d=96) == B.SP_ERR_UNSUPPORTED
    assert f(ws=None) == B.SP_ERR_WORKSPACE


def test_row_tile_counts_the_key_tiles_that_hold_an_allowed_pair():
    """sp_attn_row_tile's step counts are, by construction of the key ranges, the number of (row tile, 64-key
    tile) pairs that hold at least one allowed (query, key) pair: checked against the explicit mask."""
    import numpy as np
    from oracle import sp_attn_oracle as orc
    rng = np.random.default_rng(5)
    for _ in range(40):
        groups = []
        for _g in range(int(rng.integers(1, 4))):
            lp = int(rng.choice([0, 1, 63, 64, 65, 130, int(rng.integers(0, 500))]))
            lens = [int(rng.choice([0, 1, 32, 64, 100, int(rng.integers(0, 300))])) for _r in range(int(rng.integers(0, 5)))]
            if lp + sum(lens) == 0:
                lp = 3
            groups.append((lp, lens))
        want = {256: 0, 128: 0}
        for lp, lens in groups:
            m = orc.build_mask(lp, lens)
            T = m.shape[0]
            for bm in (256, 128):
                for t0 in range(0, T, bm):
                    for s0 in range(0, T, 64):
                        want[bm] += bool(m[t0:t0 + bm, s0:s0 + 64].any())
        pl = [g[0] for g in groups]; Gs = [len(g[1]) for g in groups]; rl = [x for g in groups for x in g[1]]
        rows, s256, s128 = B.sp_attn_row_tile(pl, Gs, rl)
        assert (s256, s128) == (want[256], want[128]), (groups, s256, s128, want)
        assert rows == (128 if 0.5 * s128 * 1.03 < s256 else 256)


def test_row_tile_rule_on_the_bench_workloads_and_the_knob():
    from paper_2511_18871_amd import workloads as W
    shape = lambda w: B.sp_attn_row_tile(w.prompt_lens(), w.Gs(), w.resp_lens_flat())[0]
    # long loops over aligned responses keep the 256-row shape; short or ragged groups take the 128-row one
    assert [shape(W.config(c)) for c in (2, 3, 4, 5, 6, 7)] == [128, 128, 256, 256, 128, 128]
    try:
        B.set_small_shape_steps(0)
        assert shape(W.config(7)) == 256
        B.set_small_shape_steps(1 << 20)
        assert shape(W.config(5)) == 128
        B.set_small_shape_steps(100)                     # threshold on the mean steps of a 256-row workgroup
        assert shape(W.config(3)) == 128 and shape(W.config(5)) == 256      # means 55 and 161
    finally:
        B.set_small_shape_steps(-1)
    assert shape(W.config(5)) == 256
    with pytest.raises(B.SpAttnError):
        B.sp_attn_row_tile([-1], [1], [5])               # a negative prompt length
