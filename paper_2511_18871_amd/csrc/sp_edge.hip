// Exact treatment of the short rows of the backward (bf16 path, gfx950).
//
// The main backward kernels round P and dS to bf16 before the second contraction.  Over a row
// with many keys those roundings average out; a row that sees a handful of keys carries weights of
// order one, so its dQ is a sum of a few large terms whose roundings do not average, and together
// with the bf16 rounding of the output they were the largest relative error of the gradients.
// The mask of Section 4.3 makes those rows easy to name: row t sees n(t) = t + 1 keys on the
// prompt and Lp + (t - st(t)) + 1 in a response, so they are the first rows of each prompt and,
// under a prompt shorter than EDGE, the first rows of each response.  For every row with
// n(t) <= EDGE this kernel recomputes, from the definitions and in fp32,
//   D = sum_s P_s dP_s      (used by the rowsum stage in place of rowsum(dO * O)), and
//   dQ = scale * sum_s dS_s K_s with dS carried into the contraction as a bf16 pair (value +
//        remainder: two MFMAs, error 2^-17); the dq pass does not store those rows.
// (The same rows' contributions to dK / dV get their remainders added inside the dkdv pass.)
//
// Work item = (segment, q head): a segment is a group's prompt or one of its responses.  An item has
// at most EDGE rows and EDGE keys, so every product is 64 x 64 x 128 or smaller; operands come
// straight from global memory in MFMA layout (no LDS): row operands as 16-byte pieces, the
// transposed operand K^T as eight 2-byte gathers per lane, 32 lanes on one row.
#include "sp_common.hpp"
#include "sp_launch.hpp"

namespace sp {
namespace {

constexpr int EDGE = EDGE_LEN;       // 64: two 32-wide MFMA blocks each way

// Segment of a response item: items enumerate the table's response-offset words (a group's G + 1
// words: its prompt's word, j = 0, then one per response); the group is the one whose words hold it.
__device__ __forceinline__ void item_segment(const int* __restrict__ tab, int n_groups, int item, int& g, int& j) {
    const int word = TAB_HEADER + TAB_GROUP_WORDS * n_groups + item;
    int lo = 0, hi = n_groups;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (tab[TAB_HEADER + TAB_GROUP_WORDS * mid + 3] <= word) lo = mid; else hi = mid;
    }
    g = lo;
    j = word - tab[TAB_HEADER + TAB_GROUP_WORDS * g + 3];
}

// value + remainder as two bf16 octets (elements e0 .. e0+7 of x)
__device__ __forceinline__ void split8(const f32x16& x, int e0, bf16x8& hi, bf16x8& lo) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const __bf16 h = (__bf16)x[e0 + i];
        hi[i] = h;
        lo[i] = (__bf16)(x[e0 + i] - (float)h);
    }
}

// Transposed operand gathered from global memory: in-lane element i is column `col` of row
// row_of(i); the 32 lanes of a half-wave read 32 consecutive columns of the same row.
template <typename RowOf>
__device__ __forceinline__ bf16x8 gather8(const __bf16* __restrict__ base, int64_t row_stride, int col, RowOf row_of) {
    bf16x8 r;
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = base[row_of(i) * row_stride + col];
    return r;
}

// ------------------------------------------------------------------------------------
// Rows that see at most EDGE keys: D, and with WITH_DQ their dQ.
// Block = (segment item, q head), two waves: wave rb owns rows 32 rb .. 32 rb + 31 of the item
// (lane c = row, S^T orientation: a lane holds one row's scores for 16 keys of a 32-key block).
// ------------------------------------------------------------------------------------
template <bool WITH_DQ>
__global__ __launch_bounds__(128) void short_rows_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                                                         const __bf16* __restrict__ v, const __bf16* __restrict__ d_o,
                                                         const float* __restrict__ lse, float* __restrict__ D,
                                                         __bf16* __restrict__ dq, int64_t T_total, int n_groups, int Hq,
                                                         int Hkv, float scale, const int* __restrict__ tab,
                                                         int response_items) {
    const int item = blockIdx.x, h = blockIdx.y;
    int g = item, j = 0;                             // prompt items: one per group, found directly
    if (response_items) {
        item_segment(tab, n_groups, item, g, j);
        if (j == 0) return;
    }
    const GroupDesc gd = load_group(tab, g);
    if (j > gd.G) return;
    const int seg0 = j == 0 ? 0 : gd.roff[j - 1], seg1 = j == 0 ? gd.Lp : gd.roff[j];
    const int base_keys = j == 0 ? 0 : gd.Lp;        // prompt keys that every row of this segment sees
    const int n_rows = min(seg1 - seg0, EDGE - base_keys);               // rows with at most EDGE keys
    const int rb = threadIdx.x >> 6, l = threadIdx.x & 63, c = l & 31, hh = l >> 5;
    if (32 * rb >= n_rows) return;
    const int n_keys = base_keys + n_rows;           // keys seen by the last of these rows
    const int kvh = h / (Hq / Hkv);
    // key number x (0 .. n_keys - 1) -> group-local token: the prompt's keys, then the segment's own
    auto key_tok = [&](int x) { x = min(x, n_keys - 1); return x < base_keys ? x : seg0 + (x - base_keys); };
    const int r = 32 * rb + c;                       // this lane's row within the segment
    const int64_t tok = gd.tok_base + seg0 + min(r, n_rows - 1);
    const __bf16* qr = q + (tok * Hq + h) * 128 + 8 * hh;
    const __bf16* gr = d_o + (tok * Hq + h) * 128 + 8 * hh;
    bf16x8 qf[8], gf[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        qf[ks] = *reinterpret_cast<const bf16x8*>(qr + 16 * ks);
        gf[ks] = *reinterpret_cast<const bf16x8*>(gr + 16 * ks);
    }
    const float L = lse[(int64_t)h * T_total + tok];
    const f32x16 zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    f32x16 P[2], dP[2];                              // per 32-key block; element e: key 32 kb + 8 (e / 4) + 4 hh + e % 4
    float acc = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
        P[kb] = zero16; dP[kb] = zero16;
        if (32 * kb >= n_keys) continue;
        const int64_t ktok = gd.tok_base + key_tok(32 * kb + c);
        const __bf16* kr = k + (ktok * Hkv + kvh) * 128 + 8 * hh;
        const __bf16* vr = v + (ktok * Hkv + kvh) * 128 + 8 * hh;
        f32x16 S = zero16;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            S = mfma32(*reinterpret_cast<const bf16x8*>(kr + 16 * ks), qf[ks], S);
            dP[kb] = mfma32(*reinterpret_cast<const bf16x8*>(vr + 16 * ks), gf[ks], dP[kb]);
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int x = 32 * kb + 8 * (e >> 2) + 4 * hh + (e & 3);
            const bool ok = r < n_rows && x <= base_keys + r;
            P[kb][e] = ok ? __expf(S[e] * scale - L) : 0.f;
            acc += P[kb][e] * dP[kb][e];
        }
    }
    const float Dr = pair_sum(acc);                  // both lanes of a row hold its D
    if (r < n_rows && hh == 0) D[(int64_t)h * T_total + tok] = Dr;
    if (!WITH_DQ) return;

    // dQ^T (d x rows) = scale * K^T (d x keys) dS^T (keys x rows), dS = P (dP - D) in fp32, fed as value + remainder
    f32x16 dqa[4] = {zero16, zero16, zero16, zero16};
    const __bf16* kcol = k + ((int64_t)gd.tok_base * Hkv + kvh) * 128 + c;
    const int64_t kv_stride = (int64_t)Hkv * 128;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
        if (32 * kb >= n_keys) continue;
        f32x16 dS;
#pragma unroll
        for (int e = 0; e < 16; ++e) dS[e] = P[kb][e] * (dP[kb][e] - Dr);
#pragma unroll
        for (int mm = 0; mm < 2; ++mm) {
            bf16x8 hi, lo;
            split8(dS, 8 * mm, hi, lo);
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                const bf16x8 A = gather8(kcol + 32 * db, kv_stride, 0, [&](int i) {
                    return (int64_t)key_tok(32 * kb + 16 * mm + 8 * (i >> 2) + 4 * hh + (i & 3)); });
                dqa[db] = mfma32(A, hi, dqa[db]);
                dqa[db] = mfma32(A, lo, dqa[db]);
            }
        }
    }
    if (r < n_rows) {
        __bf16* op = dq + (tok * Hq + h) * 128 + 4 * hh;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                bf16x4 x;
#pragma unroll
                for (int e = 0; e < 4; ++e) x[e] = (__bf16)(dqa[db][4 * gq + e] * scale);
                *reinterpret_cast<bf16x4*>(op + 32 * db + 8 * gq) = x;
            }
    }
}

}  // namespace

// D of the short rows (with_dq = false: part of the rowsum stage), or D and dQ (part of the dq stage)
hipError_t launch_short_rows(const Problem& p, bool with_dq, hipStream_t s) {
    const __bf16 *q = (const __bf16*)p.q, *k = (const __bf16*)p.k, *v = (const __bf16*)p.v, *g = (const __bf16*)p.d_o;
    auto go = [&](unsigned items, int response_items) {
        if (with_dq)
            hipLaunchKernelGGL(short_rows_kernel<true>, dim3(items, (unsigned)p.Hq), dim3(128), 0, s, q, k, v, g, p.lse,
                               p.Dbuf, (__bf16*)p.dq, p.total_tokens, p.n_groups, p.Hq, p.Hkv, p.scale, p.tab, response_items);
        else
            hipLaunchKernelGGL(short_rows_kernel<false>, dim3(items, (unsigned)p.Hq), dim3(128), 0, s, q, k, v, g, p.lse,
                               p.Dbuf, (__bf16*)nullptr, p.total_tokens, p.n_groups, p.Hq, p.Hkv, p.scale, p.tab, response_items);
    };
    // prompts: one item per group (none in response-rows mode, where prompt rows take no part)
    if (!p.resp_only) go((unsigned)p.n_groups, 0);
    // responses: their first rows qualify only under a prompt shorter than EDGE
    if (p.min_prompt_len < EDGE && p.total_responses > 0) go((unsigned)(p.n_groups + p.total_responses), 1);
    return hipGetLastError();
}

}  // namespace sp
