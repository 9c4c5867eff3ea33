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
#include <type_traits>

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

// ------------------------------------------------------------------------------------
// Software-pipelined forward.  Per key tile j a wave runs two blocks, each of which mixes
// one MFMA stream with the vector-ALU work of a DIFFERENT tile, so that both pipes are fed
// from a single instruction stream:
//   M(j): O^T += V(j-1)^T P(j-1)^T   (MFMA)   with   row max of S(j)            (VALU)
//   E(j): S(j+1) = K(j+1) Q^T        (MFMA)   with   exp2 / row sum / bf16 P(j) (VALU)
// The running-max update and the (rare) rescale of O sit between the two blocks.
// V(j) and K(j+2) are copied into LDS during iteration j, into the buffer halves that
// iteration j-1 read last.
// ------------------------------------------------------------------------------------
template <int SGB>
__global__ __launch_bounds__(512) void fwd_sw_kernel(FwdArgs a) {
    constexpr int BM = 256;
    __shared__ __attribute__((aligned(1024))) char ldsKb[2][TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char ldsVb[2][TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char ldsQ[BM * 256];          // the workgroup's query rows

    int tile, head;
    if (!decode_item(blockIdx.x, a.n_tiles, a.Hq, a.Hkv, tile, head)) return;
    int g, t0;
    find_tile(a.tab, tile, BM, g, t0);
    if (g < 0) return;
    const GroupDesc gd = load_group(a.tab, g);
    const int Lp = gd.Lp, Tg = gd.Tg;
    const int T_total = a.tab[1];

    const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), l = tid & 63;
    const int c = l & 31, hh = l >> 5, j16 = l & 15, c16 = (l >> 4) & 1;

    const int t = t0 + 32 * w + c;
    const bool valid = t < Tg;
    const int tm = valid ? t : -1;
    const int st = valid ? seg_start(gd, t) : 0;
    const int tw0 = t0 + 32 * w;
    const bool wave_valid = tw0 < Tg;
    const int tw1 = min(tw0 + 31, Tg - 1);
    const int st_first = wave_valid ? __builtin_amdgcn_readfirstlane(seg_start(gd, tw0)) : 0;
    const int st_last = wave_valid ? __builtin_amdgcn_readfirstlane(seg_start(gd, tw1)) : 0;

    // Q rows of this wave -> LDS (8 chunks of 4 rows); rows past the group's end re-read its
    // last row (their results are never stored).  B operands of S^T = K Q^T are read from here.
    {
        const __bf16* qb = a.q + ((int64_t)gd.tok_base * a.Hq + head) * 128;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int row = 32 * w + 4 * u + (l >> 4);
            const int gran = (l & 15) ^ swz(row);
            const int tq = min(t0 + row, Tg - 1);
            async_copy16(qb + (int64_t)tq * a.Hq * 128 + gran * 8, &ldsQ[(8 * w + u) * 1024]);
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
        if (it < 0 || it >= total) return;
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
        if (it < 0 || it >= total || !wave_valid) return 0;
        const int s0 = tile_at(it) * BN;
        if (a.naive) return s0 > tw1 ? 0 : 1;
        if (s0 > tw1 || (s0 >= Lp && s0 + BN <= st_first)) return 0;
        return ((s0 + BN - 1 <= tw0) && (s0 + BN <= Lp || s0 >= st_last)) ? 2 : 1;
    };

    f32x16 oacc[4], sA[2], sB[2];
    bf16x8 pb[2][2];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int mm = 0; mm < 2; ++mm) pb[kb][mm] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
    float m = -INFINITY, lsum = 0.f;
    const float cs = a.c;

    auto qk = [&](int it, f32x16 (&S)[2]) {
        const char* ldsK = ldsKb[it & 1];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) S[kb][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const bf16x8 A = lds_read_row8(ldsK, 32 * kb + c, 2 * ks + hh);
                const bf16x8 Bq = lds_read_row8(ldsQ, 32 * w + c, 2 * ks + hh);
                S[kb] = mfma32(A, Bq, S[kb]);
            }
        }
    };
    auto mask = [&](int it, f32x16 (&S)[2]) {
        const int s0 = tile_at(it) * BN;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = s0 + 32 * kb + 8 * (r >> 2) + 4 * hh + (r & 3);
                const bool ok = key <= tm && (key < Lp || key >= st);
                S[kb][r] = ok ? S[kb][r] : -INFINITY;
            }
    };
    auto rowmax = [&](const f32x16 (&S)[2]) -> float {
        float mx = S[0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, S[kb][r]);
        return pair_max(mx);
    };
    auto pv = [&](int it) {
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
    };
    auto expsum = [&](f32x16 (&S)[2]) {
        const float mc = ((m == -INFINITY) ? 0.f : m) * cs;
        float rowsum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(S[kb][r], cs, -mc));
                S[kb][r] = p;
                rowsum += p;
            }
        lsum += rowsum;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int mm = 0; mm < 2; ++mm)
                pb[kb][mm] = pack8(S[kb][8 * mm + 0], S[kb][8 * mm + 1], S[kb][8 * mm + 2],
                                   S[kb][8 * mm + 3], S[kb][8 * mm + 4], S[kb][8 * mm + 5],
                                   S[kb][8 * mm + 6], S[kb][8 * mm + 7]);
    };

    // one pipeline step for tile j: Scur holds S(j), Snext receives S(j+1)
    auto step = [&](int j, f32x16 (&Scur)[2], f32x16 (&Snext)[2]) {
        wait_vm0();
        __syncthreads();
        issue(vbase, ldsVb, j);
        issue(kbase, ldsKb, j + 2);
        const int c0 = classify(j - 1), c1 = classify(j), c2 = classify(j + 1);
        const bool fast = c0 && c1 && c2;
        if (c1 == 1) mask(j, Scur);
        float mx = -INFINITY;
        __builtin_amdgcn_sched_barrier(0);
        if (fast) {
            pv(j - 1);
            mx = rowmax(Scur);
            if (SGB) {
                __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
                }
            }
        } else {
            if (c0) pv(j - 1);
            if (c1) mx = rowmax(Scur);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (c1) {
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
        }
        __builtin_amdgcn_sched_barrier(0);
        if (fast) {
            qk(j + 1, Snext);
            expsum(Scur);
            if (SGB) {
                __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
                }
            }
        } else {
            if (c2) qk(j + 1, Snext);
            if (c1) expsum(Scur);
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    issue(kbase, ldsKb, 0);
    issue(kbase, ldsKb, 1);
    wait_vm0();
    __syncthreads();
    if (classify(0)) qk(0, sA);
    for (int j = 0; j < total; j += 2) {
        step(j, sA, sB);
        if (j + 1 < total) step(j + 1, sB, sA);
    }
    wait_vm0();
    __syncthreads();
    if (classify(total - 1)) pv(total - 1);

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
// Hand-scheduled software-pipelined forward.  Same pipeline as fwd_sw_kernel (M(j): PV of
// tile j-1 with the row max of tile j; E(j): QK of tile j+1 with the exponentials of tile
// j), but every block is written as 16 sub-blocks of {LDS read for the MFMA two steps ahead,
// one MFMA, a slice of the vector-ALU work}, fenced so the compiler keeps that order.  The
// MFMA issues every ~40 cycles and hides about five vector-ALU instructions, which is what
// each slice holds.
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(512) void fwd_mp_kernel(FwdArgs a) {
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

    const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), l = tid & 63;
    const int c = l & 31, hh = l >> 5, j16 = l & 15, c16 = (l >> 4) & 1;

    const int t = t0 + 32 * w + c;
    const bool valid = t < Tg;
    const int tm = valid ? t : -1;
    const int st = valid ? seg_start(gd, t) : 0;
    const int tw0 = t0 + 32 * w;
    const bool wave_valid = tw0 < Tg;
    const int tw1 = min(tw0 + 31, Tg - 1);
    const int st_first = wave_valid ? __builtin_amdgcn_readfirstlane(seg_start(gd, tw0)) : 0;
    const int st_last = wave_valid ? __builtin_amdgcn_readfirstlane(seg_start(gd, tw1)) : 0;

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

    auto issue = [&](const __bf16* base, char* dst, int it) {
        if (it < 0 || it >= total) return;
        const int kt = tile_at(it);
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int ci = 2 * w + u;
            const int row = 4 * ci + (l >> 4);
            const int gran = (l & 15) ^ swz(row);
            const int s = min(kt * BN + row, Tg - 1);
            async_copy16(base + (int64_t)s * kv_stride + gran * 8, dst + ci * 1024);
        }
    };
    // true when some (row, key) pair of this wave in tile `it` is masked; tiles past the end
    // of the key range (the pad step of an odd-length loop) are masked entirely
    auto needs_mask = [&](int it) -> bool {
        if (it >= total || !wave_valid || a.naive) return true;
        const int s0 = tile_at(it) * BN;
        return !((s0 + BN - 1 <= tw0) && (s0 + BN <= Lp || s0 >= st_last));
    };

    f32x16 oacc[4], sA[2], sB[2];
    unsigned pbw[16];          // P of the previous tile as packed bf16 pairs: pbw[8*kb + r/2]
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) pbw[i] = 0u;
    float m = -INFINITY, lsum = 0.f;
    const float cs = a.c;
    const f32x16 zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

    // operand fetchers, all indices compile-time
    auto ldK = [&](const char* ldsK, int i) -> bf16x8 {         // MFMA i of QK: kb = i / 8, ks = i % 8
        return lds_read_row8(ldsK, 32 * (i >> 3) + c, 2 * (i & 7) + hh);
    };
    auto ldV = [&](const char* ldsV, int i, int half) -> s16x4 { // MFMA i of PV: db = i / 4, kb = (i / 2) % 2, mm = i % 2
        const int col4 = 32 * (i >> 2) + 16 * c16 + 4 * (j16 & 3);
        const int row4 = 32 * ((i >> 1) & 1) + 16 * (i & 1) + 4 * hh + (j16 >> 2) + 8 * half;
        return lds_read_tr4(ldsV, row4, col4);
    };
    auto pbop = [&](int kb, int mm) -> bf16x8 {
        typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
        u32x4 x = {pbw[8 * kb + 4 * mm], pbw[8 * kb + 4 * mm + 1], pbw[8 * kb + 4 * mm + 2], pbw[8 * kb + 4 * mm + 3]};
        return __builtin_bit_cast(bf16x8, x);
    };
    auto pack2 = [&](float x, float y) -> unsigned {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        bf16x2 v = {(__bf16)x, (__bf16)y};
        return __builtin_bit_cast(unsigned, v);
    };

    // plain (unpipelined) pieces, used at the ends of the loop and around skipped tiles
    auto qk_plain = [&](const char* ldsK, f32x16 (&S)[2]) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
            S[i >> 3] = mfma32(ldK(ldsK, i), qreg[i & 7], (i & 7) == 0 ? zero16 : S[i >> 3]);
    };
    auto pv_plain = [&](const char* ldsV) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
            oacc[i >> 2] = mfma32(cat4(ldV(ldsV, i, 0), ldV(ldsV, i, 1)), pbop((i >> 1) & 1, i & 1), oacc[i >> 2]);
    };
    auto mask = [&](int it, f32x16 (&S)[2]) {
        const int s0 = it < total ? tile_at(it) * BN : 0;
        const int tme = it < total ? tm : -1;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = s0 + 32 * kb + 8 * (r >> 2) + 4 * hh + (r & 3);
                const bool ok = key <= tme && (key < Lp || key >= st);
                S[kb][r] = ok ? S[kb][r] : -INFINITY;
            }
    };

    // one pipeline step for tile j (parity PAR = j & 1): Scur holds S(j), Snext receives S(j+1).
    // Every wave runs every step: tiles it cannot see are handled by the mask (P = 0), the
    // first step multiplies the zero P against a zero-filled V buffer, and the last step's
    // S(j+1) is computed from a stale K buffer and never used.
    auto step = [&](int j, auto par_tag, f32x16 (&Scur)[2], f32x16 (&Snext)[2]) {
        constexpr int PAR = decltype(par_tag)::value;
        wait_vm0();
        __syncthreads();
        issue(vbase, ldsVb[PAR], j);
        issue(kbase, ldsKb[PAR], j + 2);
        const char* ldsV = ldsVb[PAR ^ 1];      // V(j-1)
        const char* ldsK = ldsKb[PAR ^ 1];      // K(j+1)
        if (needs_mask(j)) mask(j, Scur);
        __builtin_amdgcn_sched_barrier(0);
        // ---- block M: O += V(j-1) P(j-1) with the row max of S(j)
        float mx = Scur[0][0];
        {
            s16x4 ring[3][2];
            ring[0][0] = ldV(ldsV, 0, 0); ring[0][1] = ldV(ldsV, 0, 1);
            ring[1][0] = ldV(ldsV, 1, 0); ring[1][1] = ldV(ldsV, 1, 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if (i + 2 < 16) { ring[(i + 2) % 3][0] = ldV(ldsV, i + 2, 0); ring[(i + 2) % 3][1] = ldV(ldsV, i + 2, 1); }
                oacc[i >> 2] = mfma32(cat4(ring[i % 3][0], ring[i % 3][1]), pbop((i >> 1) & 1, i & 1), oacc[i >> 2]);
                mx = fmaxf(mx, fmaxf(Scur[(2 * i) >> 4][(2 * i) & 15], Scur[(2 * i + 1) >> 4][(2 * i + 1) & 15]));
                asm volatile("" : "+v"(mx));                        // keep this slice here
                __builtin_amdgcn_sched_barrier(0);
            }
        }
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
        __builtin_amdgcn_sched_barrier(0);
        // ---- block E: S(j+1) = K(j+1) Q^T with exp2 / row sum / bf16 packing of S(j)
        {
            const float mc = ((m == -INFINITY) ? 0.f : m) * cs;
            float rowsum = 0.f;
            bf16x8 ring[3];
            ring[0] = ldK(ldsK, 0);
            ring[1] = ldK(ldsK, 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if (i + 2 < 16) ring[(i + 2) % 3] = ldK(ldsK, i + 2);
                Snext[i >> 3] = mfma32(ring[i % 3], qreg[i & 7], (i & 7) == 0 ? zero16 : Snext[i >> 3]);
                const int e = 2 * i;
                const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(Scur[e >> 4][e & 15], cs, -mc));
                const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(Scur[e >> 4][(e & 15) + 1], cs, -mc));
                rowsum += p0 + p1;
                pbw[i] = pack2(p0, p1);
                asm volatile("" : "+v"(pbw[i]), "+v"(rowsum));      // keep this slice here
                __builtin_amdgcn_sched_barrier(0);
            }
            lsum += rowsum;
        }
    };

    // zero-fill the V buffer that the first step multiplies against P = 0
    for (int i = tid; i < TILE_BYTES / 16; i += 512)
        reinterpret_cast<i32x4*>(ldsVb[1])[i] = i32x4{0, 0, 0, 0};
    issue(kbase, ldsKb[0], 0);
    issue(kbase, ldsKb[1], 1);
    wait_vm0();
    __syncthreads();
    qk_plain(ldsKb[0], sA);
    const int total2 = (total + 1) & ~1;
    for (int j = 0; j < total2; j += 2) {
        step(j, std::integral_constant<int, 0>{}, sA, sB);
        step(j + 1, std::integral_constant<int, 1>{}, sB, sA);
    }
    wait_vm0();
    __syncthreads();
    pv_plain(ldsVb[1]);                    // P of step total2 - 1 (odd parity)

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
    static const int variant = getenv("SP_FWD_VARIANT") ? atoi(getenv("SP_FWD_VARIANT")) : 4;
    static const int abl = getenv("SP_ABL") ? atoi(getenv("SP_ABL")) : 0;
    if (variant == 4) hipLaunchKernelGGL(fwd_mp_kernel, dim3(grid), dim3(512), 0, s, a);
    else if (variant == 2) hipLaunchKernelGGL(fwd_sw_kernel<0>, dim3(grid), dim3(512), 0, s, a);
    else if (variant == 3) hipLaunchKernelGGL(fwd_sw_kernel<1>, dim3(grid), dim3(512), 0, s, a);
    else if (variant == 1) {
        if (abl == 0) hipLaunchKernelGGL(fwd_pp_kernel<0>, dim3(grid), dim3(512), 0, s, a);
        if (abl == 1) hipLaunchKernelGGL(fwd_pp_kernel<1>, dim3(grid), dim3(512), 0, s, a);
        if (abl == 2) hipLaunchKernelGGL(fwd_pp_kernel<2>, dim3(grid), dim3(512), 0, s, a);
        if (abl == 3) hipLaunchKernelGGL(fwd_pp_kernel<3>, dim3(grid), dim3(512), 0, s, a);
        if (abl == 4) hipLaunchKernelGGL(fwd_pp_kernel<4>, dim3(grid), dim3(512), 0, s, a);
        if (abl == 5) hipLaunchKernelGGL(fwd_pp_kernel<5>, dim3(grid), dim3(512), 0, s, a);
        if (abl == 6) hipLaunchKernelGGL(fwd_pp_kernel<6>, dim3(grid), dim3(512), 0, s, a);
    }
    else if (variant == 0)
        hipLaunchKernelGGL(fwd_kernel<NW>, dim3(grid), dim3(NW * 64), 0, s, a);
    return hipGetLastError();
}

}  // namespace sp
