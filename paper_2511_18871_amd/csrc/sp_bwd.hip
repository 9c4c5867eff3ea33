// Backward shared-prompt attention, bf16 MFMA path (gfx950).  Two deterministic passes
// after D = rowsum(dO * O):
//
//  dq pass   -- a workgroup owns a tile of query rows (like the forward) and streams the
//               keys that those rows may see: S^T = K Q^T, dP^T = V dO^T,
//               dS^T = P^T * (dP^T - D), dQ^T += K^T dS^T.
//  dkdv pass -- a workgroup owns a tile of keys of one kv head and streams every query
//               row that sees them, for each q head of the kv head: for a PROMPT key tile
//               that is the later prompt rows and all rows of all G responses, which is
//               where the prompt's dK/dV accumulate over the responses (Section 4.3,
//               grad L_shared = sum_k grad L_k).  S = Q K^T, dP = dO V^T,
//               dV^T += dO^T P, dK^T += Q^T dS.  Accumulation stays in registers, so no
//               atomics are needed and results are bitwise repeatable.
//
// The S/dP recomputation runs in both passes (7 contractions instead of 5); in exchange
// neither pass exchanges dS between lanes or accumulates through memory.
#include "sp_common.hpp"
#include "sp_launch.hpp"

namespace sp {
namespace {

constexpr int TILE_BYTES = 64 * 256;   // 64 rows x 128 bf16

struct BwdArgs {
    const __bf16* q; const __bf16* k; const __bf16* v; const __bf16* d_o;
    const float* lse; float* D; const float* L2;   // L2 = lse * log2(e), written by the rowsum stage
    __bf16* dq; __bf16* dk; __bf16* dv;
    const int* tab;
    int n_tiles, Hq, Hkv;
    float scale, c;      // c = scale * log2(e)
};

// ------------------------------------------------------------------------------------
// dq pass
// ------------------------------------------------------------------------------------
template <int NW>
__global__ __launch_bounds__(NW * 64) void bwd_dq_kernel(BwdArgs a) {
    constexpr int BM = 32 * NW, BN = 64;
    constexpr int CH = 32 / NW;                 // 1 KB chunks (4 tile rows) each wave copies per tile
    __shared__ __attribute__((aligned(1024))) char lds[2][2 * TILE_BYTES];   // [buffer][K | V]

    int tile, head;
    if (!decode_item(blockIdx.x, a.n_tiles, a.Hq, a.Hkv, tile, head)) return;
    int g, t0;
    find_tile(a.tab, tile, BM, g, t0);
    if (g < 0) return;
    const GroupDesc gd = load_group(a.tab, g);
    const int Lp = gd.Lp, Tg = gd.Tg;
    const int64_t T_total = a.tab[1];

    const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), l = tid & 63;
    const int c = l & 31, hh = l >> 5, j = l & 15, c16 = (l >> 4) & 1;

    const int t = t0 + 32 * w + c;
    const bool valid = t < Tg;
    const int tm = valid ? t : -1;
    const int st = valid ? seg_start(gd, t) : 0;
    const int tw0 = t0 + 32 * w;
    const bool wave_valid = tw0 < Tg;
    const int tw1 = min(tw0 + 31, Tg - 1);
    const int st_first = wave_valid ? seg_start(gd, tw0) : 0;
    const int st_last = wave_valid ? seg_start(gd, tw1) : 0;

    bf16x8 qreg[8], goreg[8];
    float Lq = 0.f, Dq = 0.f;
    {
        const int64_t row = ((int64_t)(gd.tok_base + (valid ? t : 0)) * a.Hq + head) * 128 + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            bf16x8 x = *reinterpret_cast<const bf16x8*>(a.q + row + 16 * ks);
            bf16x8 y = *reinterpret_cast<const bf16x8*>(a.d_o + row + 16 * ks);
            if (!valid) { x = bf16x8{0, 0, 0, 0, 0, 0, 0, 0}; y = x; }
            qreg[ks] = x; goreg[ks] = y;
        }
        if (valid) {
            Lq = a.L2[(int64_t)head * T_total + gd.tok_base + t];
            Dq = a.D[(int64_t)head * T_total + gd.tok_base + t];
        }
    }

    const int t1 = min(t0 + BM, Tg);
    int n1 = (min(Lp, t1) + BN - 1) / BN, k2b = n1, k2e = n1;
    if (t1 > Lp) {
        const int b2 = seg_start(gd, max(t0, Lp));
        k2b = max(n1, b2 / BN);
        k2e = (t1 + BN - 1) / BN;
    }
    const int total = n1 + (k2e - k2b);

    const int kvh = head / (a.Hq / a.Hkv);
    const int64_t kv_stride = (int64_t)a.Hkv * 128;
    const __bf16* kbase = a.k + ((int64_t)gd.tok_base * a.Hkv + kvh) * 128;
    const __bf16* vbase = a.v + ((int64_t)gd.tok_base * a.Hkv + kvh) * 128;

    // asynchronous tile copy global -> LDS; rows past the group's end re-read its last row
    // (those keys are always masked, the values only have to be finite)
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

    f32x16 acc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;
    const float cs = a.c;
    float dsum = 0.f;      // sum over this lane's keys of P * dP: an O-free, fp32 evaluation of D

    if (total > 0) issue_tile(tile_at(0), 0);
    for (int it = 0; it < total; ++it) {
        const int kt = tile_at(it);
        const int buf = it & 1;
        wait_vm0();
        __syncthreads();
        if (it + 1 < total) issue_tile(tile_at(it + 1), buf ^ 1);
        const char* ldsK = lds[buf];
        const char* ldsV = lds[buf] + TILE_BYTES;

        const int s0 = kt * BN;
        const bool skip = !wave_valid || s0 > tw1 || (s0 >= Lp && s0 + BN <= st_first);
        if (skip) continue;

        f32x16 sacc[2], pacc[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) { sacc[kb][r] = 0.f; pacc[kb][r] = 0.f; }
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const bf16x8 A = lds_read_row8(ldsK, 32 * kb + c, 2 * ks + hh);
                sacc[kb] = mfma32(A, qreg[ks], sacc[kb]);
            }
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const bf16x8 A = lds_read_row8(ldsV, 32 * kb + c, 2 * ks + hh);
                pacc[kb] = mfma32(A, goreg[ks], pacc[kb]);
            }
        }
        const bool full = (s0 + BN - 1 <= tw0) && (s0 + BN <= Lp || s0 >= st_last);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kb][r], cs, -Lq));
                if (!full) {
                    const int key = s0 + 32 * kb + 8 * (r >> 2) + 4 * hh + (r & 3);
                    const bool ok = key <= tm && (key < Lp || key >= st);
                    p = ok ? p : 0.f;
                }
                dsum = __builtin_fmaf(p, pacc[kb][r], dsum);
                sacc[kb][r] = p * (pacc[kb][r] - Dq);     // dS^T
            }
        bf16x8 db8[2][2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int mm = 0; mm < 2; ++mm)
                db8[kb][mm] = pack8(sacc[kb][8 * mm + 0], sacc[kb][8 * mm + 1], sacc[kb][8 * mm + 2],
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
                    const bf16x8 A = cat4(lds_read_tr4(ldsK, row4, col4), lds_read_tr4(ldsK, row4 + 8, col4));
                    acc[db] = mfma32(A, db8[kb][mm], acc[db]);
                }
        }
    }

    // D = sum_s P dP equals rowsum(dO * O) exactly, but does not inherit the bf16 rounding of O.
    // Publish it for the dkdv pass (this workgroup owns these rows of D, so overwriting is safe).
    dsum = pair_sum(dsum);
    if (valid && hh == 0) a.D[(int64_t)head * T_total + gd.tok_base + t] = dsum;
    if (valid) {
        __bf16* op = a.dq + ((int64_t)(gd.tok_base + t) * a.Hq + head) * 128 + 4 * hh;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                bf16x4 x;
#pragma unroll
                for (int e = 0; e < 4; ++e) x[e] = (__bf16)(acc[db][4 * gq + e] * a.scale);
                *reinterpret_cast<bf16x4*>(op + 32 * db + 8 * gq) = x;
            }
    }
}

// ------------------------------------------------------------------------------------
// dkdv pass
// ------------------------------------------------------------------------------------
// A workgroup of 8 waves owns 128 keys of one kv head.  Wave w works on key block kb = w & 3
// (32 keys, one per lane column) and on row half qh = w >> 2 of every 64-row query tile, so
// the two waves of a SIMD share their keys and split the rows.  K and V of the 128 keys stay
// in LDS for the whole kernel (B operands are re-read per step, which keeps a wave under 256
// registers); Q/dO tiles stream through a double buffer.  The two row halves' partial dK/dV
// are added through LDS at the end, in a fixed order.
__global__ __launch_bounds__(512) void bwd_dkdv_kernel(BwdArgs a) {
    constexpr int BNK = 128, BQ = 64;
    __shared__ __attribute__((aligned(1024))) char ldsKV[2][BNK * 256];      // [K | V] of the 128 keys
    __shared__ __attribute__((aligned(1024))) char lds[2][2 * TILE_BYTES];   // [buffer][Q | dO]
    __shared__ __attribute__((aligned(256))) float ldsLD[2][2][BQ];          // [buffer][L2 | D][row]

    int tile, kvh;
    if (!decode_item(blockIdx.x, a.n_tiles, a.Hkv, a.Hkv, tile, kvh)) return;
    // key tiles in ascending order: the first prompt tile is seen by every row (most work)
    int g, s0;
    {
        const int ng = a.tab[0];
        int base = 0;
        g = -1; s0 = 0;
        for (int gi = 0; gi < ng; ++gi) {
            const int nt = (a.tab[TAB_HEADER + TAB_GROUP_WORDS * gi + 2] + BNK - 1) / BNK;
            if (tile < base + nt) { g = gi; s0 = (tile - base) * BNK; break; }
            base += nt;
        }
    }
    if (g < 0) return;
    const GroupDesc gd = load_group(a.tab, g);
    const int Lp = gd.Lp, Tg = gd.Tg;
    const int64_t T_total = a.tab[1];

    const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), l = tid & 63;
    const int c = l & 31, hh = l >> 5, j = l & 15, c16 = (l >> 4) & 1;
    const int kb = w & 3, qh = w >> 2;

    // this lane's key (a column of S) and the rows [s, e_s) that may see it
    const int s = s0 + 32 * kb + c;
    const bool valid = s < Tg;
    const int e_s = !valid ? 0 : (s < Lp ? Tg : seg_end(gd, s));
    const int ws0 = s0 + 32 * kb;                      // wave's first key
    const bool wave_valid = ws0 < Tg;
    const int ws1 = min(ws0 + 31, Tg - 1);             // wave's last valid key
    // smallest / largest row bound e_s over the wave's keys (prompt keys: Tg; response
    // keys: the end of their response, non-decreasing in s)
    const int e_min = !wave_valid ? 0 : (ws1 < Lp ? Tg : seg_end(gd, max(ws0, Lp)));
    const int e_max = !wave_valid ? 0 : (ws0 < Lp ? Tg : seg_end(gd, ws1));

    // rows that see any key of the workgroup's tile
    const int s1 = min(s0 + BNK, Tg);
    const int row_end = s0 < Lp ? Tg : seg_end(gd, s1 - 1);
    const int qt0 = s0 / BQ, qt1 = (row_end + BQ - 1) / BQ;
    const int nqt = qt1 - qt0;
    const int rep = a.Hq / a.Hkv;
    const int total = nqt * rep;
    const int64_t q_stride = (int64_t)a.Hq * 128;
    const int64_t kv_stride = (int64_t)a.Hkv * 128;

    // K/V of the tile -> LDS (64 chunks of 4 rows; 8 per wave).  Keys past the group's end
    // re-read its last row; such lanes are masked everywhere (e_s = 0).
    {
        const __bf16* kb_ = a.k + ((int64_t)gd.tok_base * a.Hkv + kvh) * 128;
        const __bf16* vb_ = a.v + ((int64_t)gd.tok_base * a.Hkv + kvh) * 128;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int ci = w * 8 + u;                  // 0..31 K, 32..63 V
            const int row = 4 * (ci & 31) + (l >> 4);
            const int gran = (l & 15) ^ swz(row);
            const int sk = min(s0 + row, Tg - 1);
            const __bf16* src = (ci < 32 ? kb_ : vb_) + (int64_t)sk * kv_stride + gran * 8;
            async_copy16(src, &ldsKV[ci >> 5][(ci & 31) * 1024]);
        }
    }
    // Row tiles are walked from the LAST one down to the workgroup's own keys: workgroups that
    // start together (they share a kv head and an XCD) then stream the same Q/dO tiles at the
    // same time, so all but the first read of a tile hit that XCD's L2.
    // The q heads of the kv head are the inner loop, for the same reason.
    // asynchronous copy of step `it` = (row tile qt1 - 1 - it / rep, q head it % rep) into buffer `buf`.
    // Rows past the group's end re-read its last row; they are masked (t < e_s <= Tg fails).
    auto issue_tile = [&](int it, int buf) {
        const int hr = it % rep, qt = qt1 - 1 - it / rep;
        const int head = kvh * rep + hr;
        const __bf16* qb_ = a.q + ((int64_t)gd.tok_base * a.Hq + head) * 128;
        const __bf16* gb_ = a.d_o + ((int64_t)gd.tok_base * a.Hq + head) * 128;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int ci = w * 4 + u;                  // 0..15 Q, 16..31 dO
            const int row = 4 * (ci & 15) + (l >> 4);
            const int gran = (l & 15) ^ swz(row);
            const int t = min(qt * BQ + row, Tg - 1);
            const __bf16* src = (ci < 16 ? qb_ : gb_) + (int64_t)t * q_stride + gran * 8;
            async_copy16(src, &lds[buf][(ci >> 4) * TILE_BYTES + (ci & 15) * 1024]);
        }
        if (w < 2) {        // wave 0: scaled LSE of the 64 rows, wave 1: D
            const int t = min(qt * BQ + l, Tg - 1);
            const float* src = (w == 0 ? a.L2 : a.D) + (int64_t)head * T_total + gd.tok_base + t;
            async_copy4(src, reinterpret_cast<char*>(&ldsLD[buf][w][0]));
        }
    };

    f32x16 dkacc[4], dvacc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) { dkacc[db][r] = 0.f; dvacc[db][r] = 0.f; }
    const float cs = a.c;
    const char* ldsK = ldsKV[0];
    const char* ldsV = ldsKV[1];

    if (total > 0) issue_tile(0, 0);
    for (int it = 0; it < total; ++it) {
        const int qt = qt1 - 1 - it / rep;
        const int buf = it & 1;
        wait_vm0();
        __syncthreads();
        if (it + 1 < total) issue_tile(it + 1, buf ^ 1);
        const char* ldsQ = lds[buf];
        const char* ldsG = lds[buf] + TILE_BYTES;
        const float* ldsL = ldsLD[buf][0];
        const float* ldsD = ldsLD[buf][1];

        const int r0 = qt * BQ + 32 * qh;              // this wave's 32 rows
        // no row of this wave's half sees any key of this wave
        const bool skip = !wave_valid || r0 + 31 < ws0 || r0 >= e_max;
        if (skip) continue;

        f32x16 sacc, pacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) { sacc[r] = 0.f; pacc[r] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 A = lds_read_row8(ldsQ, 32 * qh + c, 2 * ks + hh);
            const bf16x8 Bk = lds_read_row8(ldsK, 32 * kb + c, 2 * ks + hh);
            sacc = mfma32(A, Bk, sacc);
        }
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 A = lds_read_row8(ldsG, 32 * qh + c, 2 * ks + hh);
            const bf16x8 Bv = lds_read_row8(ldsV, 32 * kb + c, 2 * ks + hh);
            pacc = mfma32(A, Bv, pacc);
        }
        // every row of the half sees every key of the wave
        const bool full = r0 >= ws1 && ws0 + 31 < Tg && r0 + 32 <= e_min;
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            const int rr = 32 * qh + 8 * gq + 4 * hh;
            const f32x4 L4 = *reinterpret_cast<const f32x4*>(&ldsL[rr]);
            const f32x4 D4 = *reinterpret_cast<const f32x4*>(&ldsD[rr]);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int r = 4 * gq + e;
                float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[r], cs, -L4[e]));
                if (!full) {
                    const int t = qt * BQ + rr + e;
                    p = (t >= s && t < e_s) ? p : 0.f;
                }
                sacc[r] = p;                              // P
                pacc[r] = p * (pacc[r] - D4[e]);          // dS
            }
        }
        bf16x8 p8[2], d8[2];
#pragma unroll
        for (int mm = 0; mm < 2; ++mm) {
            p8[mm] = pack8(sacc[8 * mm + 0], sacc[8 * mm + 1], sacc[8 * mm + 2], sacc[8 * mm + 3],
                           sacc[8 * mm + 4], sacc[8 * mm + 5], sacc[8 * mm + 6], sacc[8 * mm + 7]);
            d8[mm] = pack8(pacc[8 * mm + 0], pacc[8 * mm + 1], pacc[8 * mm + 2], pacc[8 * mm + 3],
                           pacc[8 * mm + 4], pacc[8 * mm + 5], pacc[8 * mm + 6], pacc[8 * mm + 7]);
        }
#pragma unroll
        for (int db = 0; db < 4; ++db) {
            const int col4 = 32 * db + 16 * c16 + 4 * (j & 3);
#pragma unroll
            for (int mm = 0; mm < 2; ++mm) {
                const int row4 = 32 * qh + 16 * mm + 4 * hh + (j >> 2);
                const bf16x8 Ag = cat4(lds_read_tr4(ldsG, row4, col4), lds_read_tr4(ldsG, row4 + 8, col4));
                dvacc[db] = mfma32(Ag, p8[mm], dvacc[db]);
                const bf16x8 Aq = cat4(lds_read_tr4(ldsQ, row4, col4), lds_read_tr4(ldsQ, row4 + 8, col4));
                dkacc[db] = mfma32(Aq, d8[mm], dkacc[db]);
            }
        }
    }

    // add the two row halves: waves 4..7 park their partial sums in LDS (the Q/dO buffers,
    // 16 KB per wave), waves 0..3 add them and write the result.  dK first, then dV.
    float* xch = reinterpret_cast<float*>(&lds[0][0]) + (size_t)kb * 4096 + l * 4;
    const int64_t orow = ((int64_t)(gd.tok_base + (valid ? s : 0)) * a.Hkv + kvh) * 128 + 4 * hh;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        f32x16* acc = pass == 0 ? dkacc : dvacc;
        __bf16* out = pass == 0 ? a.dk : a.dv;
        const float mul = pass == 0 ? a.scale : 1.0f;
        __syncthreads();
        if (qh == 1) {
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    f32x4 x = {acc[db][4 * gq], acc[db][4 * gq + 1], acc[db][4 * gq + 2], acc[db][4 * gq + 3]};
                    *reinterpret_cast<f32x4*>(xch + (db * 4 + gq) * 256) = x;
                }
        }
        __syncthreads();
        if (qh == 0 && valid) {
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const f32x4 y = *reinterpret_cast<const f32x4*>(xch + (db * 4 + gq) * 256);
                    bf16x4 x;
#pragma unroll
                    for (int e = 0; e < 4; ++e) x[e] = (__bf16)((acc[db][4 * gq + e] + y[e]) * mul);
                    *reinterpret_cast<bf16x4*>(out + orow + 32 * db + 8 * gq) = x;
                }
        }
    }
}

}  // namespace

hipError_t launch_bwd_bf16(const Problem& p, hipStream_t s) {
    hipError_t e = hipSuccess;
    if (p.stages & STAGE_ROWSUM) {
        e = launch_rowsum(p, false, s);
        if (e != hipSuccess) return e;
    }
    BwdArgs a;
    a.q = (const __bf16*)p.q; a.k = (const __bf16*)p.k; a.v = (const __bf16*)p.v; a.d_o = (const __bf16*)p.d_o;
    a.lse = p.lse; a.D = p.Dbuf; a.L2 = p.Dbuf + (int64_t)p.Hq * p.total_tokens;
    a.dq = (__bf16*)p.dq; a.dk = (__bf16*)p.dk; a.dv = (__bf16*)p.dv;
    a.tab = p.tab; a.Hq = p.Hq; a.Hkv = p.Hkv; a.scale = p.scale; a.c = p.scale * LOG2E;
    if (p.stages & STAGE_DQ) {
        constexpr int NWQ = 8;
        a.n_tiles = count_tiles(p, 32 * NWQ);
        const int grid = grid_for_items(a.n_tiles, p.Hq, p.Hkv);
        hipLaunchKernelGGL(bwd_dq_kernel<NWQ>, dim3(grid), dim3(NWQ * 64), 0, s, a);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (p.stages & STAGE_DKDV) {
        a.n_tiles = count_tiles(p, 128);
        const int grid = grid_for_items(a.n_tiles, p.Hkv, p.Hkv);
        hipLaunchKernelGGL(bwd_dkdv_kernel, dim3(grid), dim3(512), 0, s, a);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace sp
