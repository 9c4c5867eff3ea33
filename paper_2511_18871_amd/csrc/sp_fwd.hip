// Forward shared-prompt attention, bf16 MFMA path (gfx950).
//
// One workgroup owns a tile of BM consecutive packed query rows of one group and one
// q head; wave w owns 32 of those rows.  Keys/values stream through LDS in tiles of
// 64 keys.  Per tile a wave computes S^T = K Q^T (keys x queries) so that every lane
// holds scores of ONE query (column) and the online softmax needs a single
// cross-lane exchange, then O^T += V^T P^T with V read transposed from LDS.
//
// The mask of Section 4.3 (modification 3) is never materialised: with
// st(t) = first token of t's own segment (0 on the prompt),
//     allowed(t, s) = (s <= t) && (s < Lp || s >= st(t)).
// The key loop visits [0, min(Lp, t1)) and, for tiles holding response rows,
// [st(first response row), t1); everything else is wholly masked and skipped
// (the three terms of the section's complexity split).  Tiles that lie entirely in
// the allowed region skip the mask arithmetic.
#include "sp_common.hpp"
#include "sp_launch.hpp"
#include <cstdlib>

namespace sp {
namespace {

constexpr int BN = 64;                 // keys per LDS tile
constexpr int TILE_BYTES = BN * 256;   // 64 rows x 128 bf16

struct FwdArgs {
    const __bf16* q; const __bf16* k; const __bf16* v;
    __bf16* o; float* lse;
    const int* tab;
    int n_tiles, Hq, Hkv;
    float c;        // softmax_scale * log2(e)
    int naive;
};

template <int NW>
__global__ __launch_bounds__(NW * 64) void fwd_kernel(FwdArgs a) {
    constexpr int BM = 32 * NW;
    constexpr int CH = 32 / NW;                 // 1 KB chunks (4 tile rows) each wave copies per tile
    __shared__ __attribute__((aligned(1024))) char lds[2][2 * TILE_BYTES];   // [buffer][K | V]

    int tile, head;
    if (!decode_item(blockIdx.x, a.n_tiles, a.Hq, a.Hkv, tile, head)) return;
    int g, t0;
    find_tile(a.tab, tile, BM, g, t0);
    if (g < 0) return;
    const GroupDesc gd = load_group(a.tab, g);
    const int Lp = gd.Lp, Tg = gd.Tg;
    const int T_total = a.tab[1];

    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
    const int c = l & 31, hh = l >> 5, j = l & 15, c16 = (l >> 4) & 1;

    // this lane's query row, and the wave's row range
    const int t = t0 + 32 * w + c;
    const bool valid = t < Tg;
    const int tm = valid ? t : -1;
    const int st = valid ? seg_start(gd, t) : 0;
    const int tw0 = t0 + 32 * w;
    const bool wave_valid = tw0 < Tg;
    const int tw1 = min(tw0 + 31, Tg - 1);
    const int st_first = wave_valid ? seg_start(gd, tw0) : 0;
    const int st_last = wave_valid ? seg_start(gd, tw1) : 0;

    // Q as the B operand of S^T = K Q^T: column = this lane's row, 8 d-values per k-step
    bf16x8 qreg[8];
    {
        const __bf16* qp = a.q + ((int64_t)(gd.tok_base + (valid ? t : 0)) * a.Hq + head) * 128 + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            bf16x8 x = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
            if (!valid) x = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
            qreg[ks] = x;
        }
    }

    // key-tile ranges: [0, n1) and [k2b, k2e)
    const int t1 = min(t0 + BM, Tg);
    int n1, k2b, k2e;
    if (a.naive) {
        n1 = (t1 + BN - 1) / BN; k2b = k2e = n1;
    } else {
        n1 = (min(Lp, t1) + BN - 1) / BN;
        k2b = k2e = n1;
        if (t1 > Lp) {
            const int b2 = seg_start(gd, max(t0, Lp));
            k2b = max(n1, b2 / BN);
            k2e = (t1 + BN - 1) / BN;
        }
    }
    const int total = n1 + (k2e - k2b);

    const int rep = a.Hq / a.Hkv;
    const int kvh = head / rep;
    const int64_t kv_stride = (int64_t)a.Hkv * 128;
    const __bf16* kbase = a.k + ((int64_t)gd.tok_base * a.Hkv + kvh) * 128;
    const __bf16* vbase = a.v + ((int64_t)gd.tok_base * a.Hkv + kvh) * 128;

    // Asynchronous tile copy, global -> LDS.  Chunk ci (0..15 K, 16..31 V) is 4 tile rows;
    // lane i fills granule slot (i & 15) of row 4*(ci & 15) + (i >> 4), so it fetches the
    // granule that the swizzle maps to that slot.  Rows past the end of the group re-read the
    // group's last row: those keys are always masked, the values only have to be finite.
    auto issue_tile = [&](int kt, int buf) {
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int ci = w * CH + u;
            const int row = 4 * (ci & 15) + (l >> 4);
            const int gran = (l & 15) ^ swz(row);
            const int s = min(kt * BN + row, Tg - 1);
            const __bf16* src = (ci < 16 ? kbase : vbase) + (int64_t)s * kv_stride + gran * 8;
            async_copy16(src, &lds[buf][(ci >> 4) * TILE_BYTES + (ci & 15) * 1024]);
        }
    };
    auto tile_at = [&](int it) { return it < n1 ? it : k2b + (it - n1); };

    f32x16 oacc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
    float m = -INFINITY, lsum = 0.f;
    const float cs = a.c;

    if (total > 0) issue_tile(tile_at(0), 0);
    for (int it = 0; it < total; ++it) {
        const int kt = tile_at(it);
        const int buf = it & 1;
        wait_vm0();            // this wave's share of tile `it` has landed
        __syncthreads();       // everyone's has; everyone is done reading the other buffer
        if (it + 1 < total) issue_tile(tile_at(it + 1), buf ^ 1);
        const char* ldsK = lds[buf];
        const char* ldsV = lds[buf] + TILE_BYTES;

        const int s0 = kt * BN;
        const bool skip = !wave_valid || s0 > tw1 ||
                          (!a.naive && s0 >= Lp && s0 + BN <= st_first);
        if (skip) continue;

        f32x16 sacc[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[kb][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const bf16x8 A = lds_read_row8(ldsK, 32 * kb + c, 2 * ks + hh);
                sacc[kb] = mfma32(A, qreg[ks], sacc[kb]);
            }
        }
        const bool full = !a.naive && (s0 + BN - 1 <= tw0) && (s0 + BN <= Lp || s0 >= st_last);
        if (!full) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = s0 + 32 * kb + 8 * (r >> 2) + 4 * hh + (r & 3);
                    const bool ok = key <= tm && (key < Lp || key >= st);
                    sacc[kb][r] = ok ? sacc[kb][r] : -INFINITY;
                }
        }
        float mx = sacc[0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[kb][r]);
        mx = pair_max(mx);
        const float mnew = fmaxf(m, mx);
        if (__builtin_amdgcn_ballot_w64(mnew > m) != 0) {      // some row's running max grew
            const float muse = (mnew == -INFINITY) ? 0.f : mnew;
            const float alpha = __builtin_amdgcn_exp2f((m - muse) * cs);
            lsum *= alpha;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
            m = mnew;
        }
        const float mc = ((m == -INFINITY) ? 0.f : m) * cs;
        float rowsum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kb][r], cs, -mc));
                sacc[kb][r] = p;
                rowsum += p;
            }
        lsum += rowsum;

        bf16x8 pb[2][2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int mm = 0; mm < 2; ++mm)
                pb[kb][mm] = pack8(sacc[kb][8 * mm + 0], sacc[kb][8 * mm + 1], sacc[kb][8 * mm + 2],
                                   sacc[kb][8 * mm + 3], sacc[kb][8 * mm + 4], sacc[kb][8 * mm + 5],
                                   sacc[kb][8 * mm + 6], sacc[kb][8 * mm + 7]);
#pragma unroll
        for (int db = 0; db < 4; ++db) {
            const int col4 = 32 * db + 16 * c16 + 4 * (j & 3);
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int mm = 0; mm < 2; ++mm) {
                    const int row4 = 32 * kb + 16 * mm + 4 * hh + (j >> 2);
                    const bf16x8 A = cat4(lds_read_tr4(ldsV, row4, col4),
                                          lds_read_tr4(ldsV, row4 + 8, col4));
                    oacc[db] = mfma32(A, pb[kb][mm], oacc[db]);
                }
        }
    }

    // epilogue: O = acc / l, LSE = (m*c + log2 l) * ln 2
    const float ltot = pair_sum(lsum);
    if (valid) {
        const float inv = 1.0f / ltot;
        __bf16* op = a.o + ((int64_t)(gd.tok_base + t) * a.Hq + head) * 128 + 4 * hh;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                bf16x4 x;
#pragma unroll
                for (int e = 0; e < 4; ++e) x[e] = (__bf16)(oacc[db][4 * gq + e] * inv);
                *reinterpret_cast<bf16x4*>(op + 32 * db + 8 * gq) = x;
            }
        if (hh == 0)
            a.lse[(int64_t)head * T_total + gd.tok_base + t] = (m * cs + __log2f(ltot)) * LN2;
    }
}

// ------------------------------------------------------------------------------------
// Ping-pong forward: 8 waves, the two waves that share a SIMD run half an iteration apart.
// Per key tile j a wave alternates between two clusters separated by workgroup barriers:
//   Y(j)   softmax of S(j): mask, running max, exp2, row sum, bf16 P          (VALU)
//   X(j+1) O^T += V(j)^T P(j)^T, then S(j+1) = K(j+1) Q^T                       (MFMA)
// Waves 4..7 enter the sequence one barrier later than waves 0..3, so while one wave of a
// SIMD issues MFMAs the other issues the softmax arithmetic.  Tile copies K(j+2), V(j+1) are
// issued two barriers before their first use into the buffer halves that were last read
// two barriers earlier.
// ------------------------------------------------------------------------------------
template <int ABL>
__global__ __launch_bounds__(512) void fwd_pp_kernel(FwdArgs a) {
    constexpr int BM = 256;
    __shared__ __attribute__((aligned(1024))) char ldsKb[2][TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char ldsVb[2][TILE_BYTES];

    int tile, head;
    if (!decode_item(blockIdx.x, a.n_tiles, a.Hq, a.Hkv, tile, head)) return;
    int g, t0;
    find_tile(a.tab, tile, BM, g, t0);
    if (g < 0) return;
    const GroupDesc gd = load_group(a.tab, g);
    const int Lp = gd.Lp, Tg = gd.Tg;
    const int T_total = a.tab[1];

    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
    const int c = l & 31, hh = l >> 5, j16 = l & 15, c16 = (l >> 4) & 1;
    const int grp = (ABL == 5) ? (w & 1) : (ABL == 6) ? ((w >> 1) & 1) : (w >> 2);

    const int t = t0 + 32 * w + c;
    const bool valid = t < Tg;
    const int tm = valid ? t : -1;
    const int st = valid ? seg_start(gd, t) : 0;
    const int tw0 = t0 + 32 * w;
    const bool wave_valid = tw0 < Tg;
    const int tw1 = min(tw0 + 31, Tg - 1);
    const int st_first = wave_valid ? seg_start(gd, tw0) : 0;
    const int st_last = wave_valid ? seg_start(gd, tw1) : 0;

    bf16x8 qreg[8];
    {
        const __bf16* qp = a.q + ((int64_t)(gd.tok_base + (valid ? t : 0)) * a.Hq + head) * 128 + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            bf16x8 x = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
            if (!valid) x = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
            qreg[ks] = x;
        }
    }

    const int t1 = min(t0 + BM, Tg);
    int n1, k2b, k2e;
    if (a.naive) {
        n1 = (t1 + BN - 1) / BN; k2b = k2e = n1;
    } else {
        n1 = (min(Lp, t1) + BN - 1) / BN;
        k2b = k2e = n1;
        if (t1 > Lp) {
            const int b2 = seg_start(gd, max(t0, Lp));
            k2b = max(n1, b2 / BN);
            k2e = (t1 + BN - 1) / BN;
        }
    }
    const int total = n1 + (k2e - k2b);
    auto tile_at = [&](int it) { return it < n1 ? it : k2b + (it - n1); };

    const int kvh = head / (a.Hq / a.Hkv);
    const int64_t kv_stride = (int64_t)a.Hkv * 128;
    const __bf16* kbase = a.k + ((int64_t)gd.tok_base * a.Hkv + kvh) * 128;
    const __bf16* vbase = a.v + ((int64_t)gd.tok_base * a.Hkv + kvh) * 128;

    // each wave copies chunks 2w, 2w+1 (4 rows each) of a 64-row tile
    auto issue = [&](const __bf16* base, char (*dst)[TILE_BYTES], int it) {
        if (it >= total) return;
        const int kt = tile_at(it);
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int ci = 2 * w + u;
            const int row = 4 * ci + (l >> 4);
            const int gran = (l & 15) ^ swz(row);
            const int s = min(kt * BN + row, Tg - 1);
            async_copy16(base + (int64_t)s * kv_stride + gran * 8, &dst[it & 1][ci * 1024]);
        }
    };
    // 0 = no row of this wave sees the tile, 1 = element mask needed, 2 = fully visible
    auto classify = [&](int it) -> int {
        if (it >= total || !wave_valid) return 0;
        const int s0 = tile_at(it) * BN;
        if (a.naive) return s0 > tw1 ? 0 : 1;
        if (s0 > tw1 || (s0 >= Lp && s0 + BN <= st_first)) return 0;
        return ((s0 + BN - 1 <= tw0) && (s0 + BN <= Lp || s0 >= st_last)) ? 2 : 1;
    };

    f32x16 oacc[4], sacc[2];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
    float m = -INFINITY, lsum = 0.f;
    const float cs = a.c;

    auto qk = [&](int it) {
        const char* ldsK = ldsKb[it & 1];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[kb][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const bf16x8 A = lds_read_row8(ldsK, 32 * kb + c, 2 * ks + hh);
                sacc[kb] = mfma32(A, qreg[ks], sacc[kb]);
            }
        }
    };

    issue(kbase, ldsKb, 0); issue(vbase, ldsVb, 0); issue(kbase, ldsKb, 1);
    wait_vm0();
    __syncthreads();
    if (grp == 1) { __builtin_amdgcn_s_barrier(); }
    __builtin_amdgcn_sched_barrier(0);
    if (classify(0)) qk(0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);

    for (int it = 0; it < total; ++it) {
        const int cls = classify(it);
        bf16x8 pb[2][2];
        // ---------------- Y(it): softmax ----------------
        if (grp == 1) { issue(kbase, ldsKb, it + 2); issue(vbase, ldsVb, it + 1); }
        if (cls && ABL != 2) {
            if (cls == 1) {
                const int s0 = tile_at(it) * BN;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = s0 + 32 * kb + 8 * (r >> 2) + 4 * hh + (r & 3);
                        const bool ok = key <= tm && (key < Lp || key >= st);
                        sacc[kb][r] = ok ? sacc[kb][r] : -INFINITY;
                    }
            }
            float mx = sacc[0][0];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[kb][r]);
            mx = pair_max(mx);
            const float mnew = fmaxf(m, mx);
            if (__builtin_amdgcn_ballot_w64(mnew > m) != 0) {
                const float muse = (mnew == -INFINITY) ? 0.f : mnew;
                const float alpha = __builtin_amdgcn_exp2f((m - muse) * cs);
                lsum *= alpha;
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
                m = mnew;
            }
            const float mc = ((m == -INFINITY) ? 0.f : m) * cs;
            float rowsum = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float x = __builtin_fmaf(sacc[kb][r], cs, -mc);
                    const float p = (ABL == 1) ? x : __builtin_amdgcn_exp2f(x);
                    sacc[kb][r] = p;
                    rowsum += p;
                }
            lsum += rowsum;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int mm = 0; mm < 2; ++mm)
                    pb[kb][mm] = pack8(sacc[kb][8 * mm + 0], sacc[kb][8 * mm + 1], sacc[kb][8 * mm + 2],
                                       sacc[kb][8 * mm + 3], sacc[kb][8 * mm + 4], sacc[kb][8 * mm + 5],
                                       sacc[kb][8 * mm + 6], sacc[kb][8 * mm + 7]);
        }
        if (grp == 0) wait_vm0();
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        // ---------------- X(it+1): PV(it), then QK(it+1) ----------------
        if (grp == 0) { issue(kbase, ldsKb, it + 2); issue(vbase, ldsVb, it + 1); }
        __builtin_amdgcn_s_setprio(1);
        if (cls && ABL != 3) {
            const char* ldsV = ldsVb[it & 1];
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                const int col4 = 32 * db + 16 * c16 + 4 * (j16 & 3);
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int mm = 0; mm < 2; ++mm) {
                        const int row4 = 32 * kb + 16 * mm + 4 * hh + (j16 >> 2);
                        const bf16x8 A = cat4(lds_read_tr4(ldsV, row4, col4),
                                              lds_read_tr4(ldsV, row4 + 8, col4));
                        oacc[db] = mfma32(A, pb[kb][mm], oacc[db]);
                    }
            }
        }
        if (classify(it + 1) && ABL != 4) qk(it + 1);
        __builtin_amdgcn_s_setprio(0);
        if (grp == 1) wait_vm0();
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    }
    if (grp == 0) { __builtin_amdgcn_s_barrier(); }

    const float ltot = pair_sum(lsum);
    if (valid) {
        const float inv = 1.0f / ltot;
        __bf16* op = a.o + ((int64_t)(gd.tok_base + t) * a.Hq + head) * 128 + 4 * hh;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                bf16x4 x;
#pragma unroll
                for (int e = 0; e < 4; ++e) x[e] = (__bf16)(oacc[db][4 * gq + e] * inv);
                *reinterpret_cast<bf16x4*>(op + 32 * db + 8 * gq) = x;
            }
        if (hh == 0)
            a.lse[(int64_t)head * T_total + gd.tok_base + t] = (m * cs + __log2f(ltot)) * LN2;
    }
}

}  // namespace

hipError_t launch_fwd_bf16(const Problem& p, hipStream_t s) {
    FwdArgs a;
    a.q = (const __bf16*)p.q; a.k = (const __bf16*)p.k; a.v = (const __bf16*)p.v;
    a.o = (__bf16*)p.o_out; a.lse = p.lse_out; a.tab = p.tab;
    a.Hq = p.Hq; a.Hkv = p.Hkv; a.c = p.scale * LOG2E; a.naive = p.naive;
    constexpr int NW = 8;
    a.n_tiles = count_tiles(p, 32 * NW);
    const int grid = grid_for_items(a.n_tiles, p.Hq, p.Hkv);
    static const int variant = getenv("SP_FWD_VARIANT") ? atoi(getenv("SP_FWD_VARIANT")) : 1;
    static const int abl = getenv("SP_ABL") ? atoi(getenv("SP_ABL")) : 0;
    if (variant == 1) {
        if (abl == 0) hipLaunchKernelGGL(fwd_pp_kernel<0>, dim3(grid), dim3(512), 0, s, a);
        if (abl == 1) hipLaunchKernelGGL(fwd_pp_kernel<1>, dim3(grid), dim3(512), 0, s, a);
        if (abl == 2) hipLaunchKernelGGL(fwd_pp_kernel<2>, dim3(grid), dim3(512), 0, s, a);
        if (abl == 3) hipLaunchKernelGGL(fwd_pp_kernel<3>, dim3(grid), dim3(512), 0, s, a);
        if (abl == 4) hipLaunchKernelGGL(fwd_pp_kernel<4>, dim3(grid), dim3(512), 0, s, a);
        if (abl == 5) hipLaunchKernelGGL(fwd_pp_kernel<5>, dim3(grid), dim3(512), 0, s, a);
        if (abl == 6) hipLaunchKernelGGL(fwd_pp_kernel<6>, dim3(grid), dim3(512), 0, s, a);
    }
    else
        hipLaunchKernelGGL(fwd_kernel<NW>, dim3(grid), dim3(NW * 64), 0, s, a);
    return hipGetLastError();
}

}  // namespace sp
