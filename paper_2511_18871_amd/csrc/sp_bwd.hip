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
#include <type_traits>

namespace sp {
namespace {

constexpr int TILE_BYTES = 64 * 256;   // 64 rows x 128 bf16

struct BwdArgs {
    const __bf16* q; const __bf16* k; const __bf16* v; const __bf16* d_o;
    const float* lse; float* D; float* L2;         // L2 = lse * log2(e), written by the rowsum stage (or the dq pass, below)
    // dq pass with the rowsum stage folded in: D = rowsum(dO * (o + residual)) is formed in the prologue from
    // the dO rows the pass loads anyway, and the D / L2 planes are written for the dkdv pass
    int fused_rowsum;
    const __bf16* o; const __bf16* o_lo; const uint32_t* lo_flag;
    __bf16* dq; __bf16* dk; __bf16* dv;
    const int* tab;
    Schedule sched;      // tile descriptors and per-token segment bounds, written by the schedule kernel of the call
    int n_tiles, n_groups, Hq, Hkv;
    float scale, c;      // c = scale * log2(e)
    int resp_only;       // only response rows are computed (dq) / contribute (dk, dv)
    int accumulate;      // dk, dv are added to what the output buffers hold
    // dkdv pass on small problems: one workgroup per (key tile, Q head) instead of per (key tile,
    // kv head); the per-q-head partial sums go to `partial` in fp32 and a second kernel adds them
    int head_split;
    float* partial;      // [2 (dK, dV)][rep][T_total][Hkv][128] fp32
};

// ------------------------------------------------------------------------------------
// dq pass
// ------------------------------------------------------------------------------------
//
// Two shapes of workgroup, as in the forward.  NW = 8: 256 rows, a ring of three slots of a whole 64-key tile
// (K and V: 96 KB), one workgroup per CU, one barrier per tile.  NW = 4: 128 rows, a ring of four slots of HALF
// a tile (32 keys of K and V: 64 KB), one barrier per half, two workgroups per CU: for packings whose key
// loops are short, where a workgroup's fixed costs (a quarter of its life with one workgroup per CU) then
// overlap with the other workgroup's loop and fewer rows ride along through tiles they cannot see.
template <int NW>
__global__ __launch_bounds__(NW * 64, 2) void bwd_dq_kernel(BwdArgs a) {
    constexpr int BM = 32 * NW, BN = 64;
    constexpr int RD = 3;                       // LDS operand ring depth (prefetch distance RD - 1 MFMAs)
    constexpr int NE1 = 5;                      // elements of a half's vector work done under the previous D stage
    static_assert(NW == 8 || NW == 4, "the copy split below assumes eight or four waves");
    constexpr int NSLOT = NW == 8 ? 3 : 4;
    constexpr int SLOT_BYTES = NW == 8 ? 2 * TILE_BYTES : TILE_BYTES;       // [K | V] of 64 keys, or of 32
    constexpr int V_OFF = SLOT_BYTES / 2;                                    // where V starts inside a slot
    __shared__ __attribute__((aligned(1024))) char lds[NSLOT][SLOT_BYTES];

    int tile, head;
    if (!decode_item(blockIdx.x, a.n_tiles, a.Hq, a.Hkv, tile, head)) return;
    const TileDesc td = (BM == 256 ? a.sched.tiles256 : a.sched.tiles128)[tile];
    const int ti = td.ti;
    GroupDesc gd;
    gd.tok_base = td.tok_base; gd.Lp = td.Lp; gd.Tg = td.Tg; gd.G = 0; gd.roff = nullptr;
    const int Lp = gd.Lp, Tg = gd.Tg;
    const int t0 = ((Tg + BM - 1) / BM - 1 - ti) * BM;   // a group's last tile first: it carries the most work
    const int64_t T_total = a.tab[1];
    if (a.resp_only && t0 + BM <= Lp) return;      // a tile of prompt rows only

    const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), l = tid & 63;
    const int c = l & 31, hh = l >> 5, j = l & 15, c16 = (l >> 4) & 1;

    const int t = t0 + 32 * w + c;
    const bool valid = t < Tg;
    const int tm = valid ? t : -1;
    const int tw0 = t0 + 32 * w;
    const bool wave_valid = tw0 < Tg;
    const int tw1 = min(tw0 + 31, Tg - 1);
    // first own-segment key of this lane's row and of the workgroup's first response row (0 on the prompt)
    const int st = valid ? a.sched.key_lo[gd.tok_base + t] : 0;
    const int b2 = __builtin_amdgcn_readfirstlane(a.sched.key_lo[gd.tok_base + min(max(t0, Lp), Tg - 1)]);
    // lanes 0..31 hold the wave's rows in order: the last valid row's start comes from its lane
    const int st_last = wave_valid ? __builtin_amdgcn_readlane(st, tw1 - tw0) : 0;

    auto sgpr64 = [](const void* p) -> uint64_t {
        const uint64_t b = (uint64_t)(uintptr_t)p;
        return ((uint64_t)(unsigned)__builtin_amdgcn_readfirstlane((int)(b >> 32)) << 32) |
               (uint64_t)(unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)b);
    };
    auto lds_u32 = [](char* p) -> unsigned {
        return __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)p);
    };

    // The wave's rows of q and dO (and of o and its residual for the folded rowsum) in MFMA operand layout.
    // Loaded straight from memory in that layout an instruction touches 32 rows and uses 32 bytes of each,
    // and the 32 such instructions of a wave are bound by the address unit: a quarter of a 128-row workgroup's
    // life on short key loops.  They come in like the K/V tiles instead: copied row-contiguous (four whole
    // rows per instruction) into the wave's own share of the not yet used tile ring, swizzled, and read back
    // with the operand reads of a K tile.  The share holds TPR tensors of 32 rows at a time.  Rows past the
    // end of the group read the group's last row: their scores are all masked (P = dS = 0 whatever q and dO
    // hold, and a non-finite dO there only reaches dq rows that are not stored).
    constexpr int SHARE = NSLOT * SLOT_BYTES / NW;          // 16 KB (NW = 4), 12 KB (NW = 8)
    constexpr int TPR = SHARE / 8192;
    char* const stg = &lds[0][0] + SHARE * w;
    const int rbase = min(tw0, Tg - 1), rlast = Tg - 1 - rbase;
    auto stage_rows = [&](const __bf16* tensor, int slot) {
        const uint64_t sb = sgpr64(tensor + ((int64_t)(gd.tok_base + rbase) * a.Hq + head) * 128);
        const unsigned m0 = lds_u32(stg) + 8192u * slot;
        const unsigned row_bytes = (unsigned)a.Hq * 256u;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int row = 4 * u + (l >> 4);
            async_copy16_sm(sb, (unsigned)min(row, rlast) * row_bytes + (((l & 15) ^ swz(row)) << 4), m0 + 1024u * u);
        }
    };
    auto read_rows = [&](int slot, bf16x8 (&r)[8]) {
        asm volatile("" ::: "memory");              // the reads stay behind the wait for the copies
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) r[ks] = lds_read_row8(stg + 8192 * slot, c, 2 * ks + hh);
    };
    auto lds_reads_done = [] { __builtin_amdgcn_s_waitcnt(0xC07F); };     // lgkmcnt(0): the share may be overwritten

    bf16x8 qreg[8], goreg[8];
    float Lq = 0.f, Dq = 0.f;
    {
        // whether the forward's rounding residual is valid: one word, read ahead of the copies so that its wait
        // is theirs
        const bool use_lo = a.fused_rowsum && a.o_lo != nullptr &&
                            (a.lo_flag == nullptr || __builtin_amdgcn_readfirstlane((int)*a.lo_flag) != 0);
        float lse_row = 0.f;
        if (a.fused_rowsum) {
            if (valid) lse_row = a.lse[(int64_t)head * T_total + gd.tok_base + t];
        } else if (valid) {
            Lq = a.L2[(int64_t)head * T_total + gd.tok_base + t];
            Dq = a.D[(int64_t)head * T_total + gd.tok_base + t];
        }
        stage_rows(a.q, 0);
        if constexpr (TPR == 2) {
            stage_rows(a.d_o, 1);
            wait_vm0();
            read_rows(0, qreg);
            read_rows(1, goreg);
        } else {
            wait_vm0();
            read_rows(0, qreg);
            lds_reads_done();
            stage_rows(a.d_o, 0);
            wait_vm0();
            read_rows(0, goreg);
        }
        if (a.fused_rowsum) {
            // The arithmetic of rowsum_bf16_kernel, operation for operation, so that a backward in one call
            // and a staged one agree bit for bit: that kernel gives a row to 16 lanes of 8 elements each
            // (lane `sub` = elements 8 sub .. 8 sub + 7, summed in order by fma) and adds the lanes in an
            // xor-shuffle tree (8, 4, 2, 1).  This lane holds the chunks sub = 2 ks + hh, so the first three
            // levels are sums inside the lane and the last one is the exchange with the row's other lane.
            bf16x8 oreg[8], lreg[8];
            lds_reads_done();
            stage_rows(a.o, 0);
            if constexpr (TPR == 2) {
                if (use_lo) stage_rows(a.o_lo, 1);
                wait_vm0();
                read_rows(0, oreg);
                if (use_lo) read_rows(1, lreg);
            } else {
                wait_vm0();
                read_rows(0, oreg);
                if (use_lo) {
                    lds_reads_done();
                    stage_rows(a.o_lo, 0);
                    wait_vm0();
                    read_rows(0, lreg);
                }
            }
            float ch[8];
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                float acc1 = 0.f;
                if (use_lo) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc1 = __builtin_fmaf((float)goreg[ks][e], (float)oreg[ks][e] + (float)lreg[ks][e], acc1);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc1 = __builtin_fmaf((float)goreg[ks][e], (float)oreg[ks][e], acc1);
                }
                ch[ks] = acc1;
            }
            const float x0 = ch[0] + ch[4], x1 = ch[1] + ch[5], x2 = ch[2] + ch[6], x3 = ch[3] + ch[7];
            const float y0 = x0 + x2, y1 = x1 + x3;
            Dq = pair_sum(y0 + y1);
            if (valid) {
                Lq = lse_row * LOG2E;
                if (hh == 0) a.L2[(int64_t)head * T_total + gd.tok_base + t] = Lq;
            } else {
                Dq = 0.f;
            }
        }
        // the shares overlap the ring slots that the first tile copies (of other waves, too) are about to fill
        lds_reads_done();
        __syncthreads();
    }

    const int t1 = min(t0 + BM, Tg);
    int n1 = (min(Lp, t1) + BN - 1) / BN, k2b = n1, k2e = n1;
    if (t1 > Lp) {
        k2b = max(n1, b2 / BN);
        k2e = (t1 + BN - 1) / BN;
    }
    const int total = n1 + (k2e - k2b);

    const int kvh = head / (a.Hq / a.Hkv);
    const int64_t kv_stride = (int64_t)a.Hkv * 128;
    const __bf16* kbase = a.k + ((int64_t)gd.tok_base * a.Hkv + kvh) * 128;
    const __bf16* vbase = a.v + ((int64_t)gd.tok_base * a.Hkv + kvh) * 128;

    // Tile copy global -> LDS, issued by the first wave of each SIMD (w < 4): those waves are
    // served first by the instruction arbiter and would otherwise idle at the barrier.  Wave w
    // copies chunks 4w .. 4w+3 (4 rows each) of the K tile and of the V tile.  Rows past the
    // group's end re-read its last row (those keys are always masked; values must be finite).
    const unsigned stride_b = (unsigned)(kv_stride * 2);
    // (NW = 4: every wave is the first of its SIMD within the workgroup; wave w copies chunks 2w, 2w+1 of the
    // 32 rows of K and of V of a half.)
    const bool copier = w < 4;
    constexpr int NCH = NW == 8 ? 4 : 2;        // chunks of K (and of V) a copying wave moves per slot
    unsigned voff[NCH];
#pragma unroll
    for (int u = 0; u < NCH; ++u) {
        const int row = 4 * (NCH * (w & 3) + u) + (l >> 4);
        voff[u] = row * stride_b + (((l & 15) ^ swz(row)) << 4);
    }
    const uint64_t kbase_s = sgpr64(kbase), vbase_s = sgpr64(vbase);
    unsigned m0slot[NSLOT];
#pragma unroll
    for (int i = 0; i < NSLOT; ++i) m0slot[i] = lds_u32(lds[i]) + 1024u * NCH * (w & 3);
    auto tile_at = [&](int it) { return it < n1 ? it : k2b + (it - n1); };
    // NW = 8: `it` counts 64-key tiles; NW = 4: halves of them (32 keys), each into a slot of its own
    auto issue = [&](int it, int slot) {
        if (!copier || it >= (NW == 8 ? total : 2 * total)) return;
        // first key of the slot; the second half of a group's last tile may lie wholly past the group's end: it
        // is then read from the group's last row on (every offset below stays non-negative)
        const int key0 = min(NW == 8 ? tile_at(it) * BN : tile_at(it >> 1) * BN + 32 * (it & 1), Tg - 1);
        constexpr int ROWS = NW == 8 ? BN : 32;
        const uint64_t off = (uint64_t)(unsigned)key0 * stride_b;
        const unsigned m0 = m0slot[slot];
        if (key0 + ROWS <= Tg) {
#pragma unroll
            for (int u = 0; u < NCH; ++u) async_copy16_sm(kbase_s + off, voff[u], m0 + 1024u * u);
#pragma unroll
            for (int u = 0; u < NCH; ++u) async_copy16_sm(vbase_s + off, voff[u], m0 + V_OFF + 1024u * u);
        } else {
            const int last = Tg - 1 - key0;
#pragma unroll
            for (int u = 0; u < NCH; ++u) {
                const int row = 4 * (NCH * (w & 3) + u) + (l >> 4);
                const unsigned vo = min(row, last) * stride_b + (((l & 15) ^ swz(row)) << 4);
                async_copy16_sm(kbase_s + off, vo, m0 + 1024u * u);
                async_copy16_sm(vbase_s + off, vo, m0 + V_OFF + 1024u * u);
            }
        }
    };

    f32x16 acc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;
    const float cs = a.c;
    float dsum = 0.f;      // sum over this lane's keys of P * dP: an O-free, fp32 evaluation of D
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    // Work is cut into halves of 32 keys (two per 64-key tile).  For half h a wave runs
    //   M(h): S^T, dP^T of the half (16 MFMAs);  V(h): P^T = exp2(S^T c - L), dS^T = P^T (dP^T - D)
    //   (16 elements of vector work);  D(h): dQ^T += K^T dS^T (8 MFMAs),
    // software-pipelined so that the vector work always sits between MFMAs of other halves:
    // V(h) is spread over the slices of D(h-1) (its first NE1 elements) and M(h+1) (the rest).
    // Each slice is {LDS read for the MFMA RD-1 ahead, one MFMA, a piece of vector work}, fenced.
    // Masking is done beforehand on S (masked score = -inf gives P = 0 and dS = 0), so the
    // pipeline body is the same for every tile; the half past the last one is masked whole.
    const int H = 2 * total;
    auto s0_of = [&](int h) { return tile_at(h >> 1) * BN + 32 * (h & 1); };
    auto needs_mask = [&](int h) -> bool {
        if (h >= H || !wave_valid) return true;
        const int s0 = s0_of(h);
        return !((s0 + 31 <= tw0) && (s0 + 32 <= Lp || s0 >= st_last));
    };
    auto mask = [&](int h, f32x16& S, f32x16& P) {
        const bool none = h >= H;
        const int s0 = none ? 0 : s0_of(h);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = s0 + 8 * (r >> 2) + 4 * hh + (r & 3);
            const bool ok = !none && key <= tm && (key < Lp || key >= st);
            S[r] = ok ? S[r] : -INFINITY;
            P[r] = none ? 0.f : P[r];
        }
    };
    auto ldm = [&](const char* slot, int half, int i) {      // operand i of M: K rows for i < 8 (S), V rows after (dP)
        return lds_read_row8(slot + ((i & 8) ? V_OFF : 0), 32 * half + c, 2 * (i & 7) + hh);
    };
    auto ldd = [&](const char* slot, int half, int i, int part) {   // MFMA i of D: db = i / 2, 16-key step mm = i % 2
        const int col4 = 32 * (i >> 1) + 16 * c16 + 4 * (j & 3);
        const int row4 = 32 * half + 16 * (i & 1) + 4 * hh + (j >> 2);
        return lds_read_tr4(slot, row4 + 8 * part, col4);
    };
    auto pack2 = [&](float x, float y) -> unsigned {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        bf16x2 v = {(__bf16)x, (__bf16)y};
        return __builtin_bit_cast(unsigned, v);
    };
    float tprev = 0.f;
    // vector work on element r: the exponential is issued in one slice and consumed in the next
    auto v_issue = [&](f32x16& S, int r) {
        const float tcur = __builtin_amdgcn_exp2f(__builtin_fmaf(S[r], cs, -Lq));
        return tcur;
    };
    auto v_consume = [&](f32x16& S, f32x16& P, int r, float p) {
        dsum = __builtin_fmaf(p, P[r], dsum);
        S[r] = p * (P[r] - Dq);
        asm volatile("" : "+v"(dsum), "+v"(S[r]));
    };
    // One pipeline stage for half h: Sc/Pc hold S, dP of half h (elements < NE1 already turned
    // into dS), Sn/Pn receive half h+1.
    auto stage = [&](int h, f32x16& Sc, f32x16& Pc, f32x16& Sn, f32x16& Pn,
                     const char* slotM, int halfM, const char* slotD, int halfD) {
        unsigned pk[8];
        {   // M(h+1) with the rest of V(h)
            bf16x8 ring[RD];
#pragma unroll
            for (int i = 0; i < RD - 1; ++i) ring[i] = ldm(slotM, halfM, i);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if (i + RD - 1 < 16) ring[(i + RD - 1) % RD] = ldm(slotM, halfM, i + RD - 1);
                if (i & 8) Pn = mfma32(ring[i % RD], goreg[i & 7], i == 8 ? zero16 : Pn);
                else Sn = mfma32(ring[i % RD], qreg[i & 7], i == 0 ? zero16 : Sn);
                float tcur = 0.f;
                if (NE1 + i < 16) { tcur = v_issue(Sc, NE1 + i); asm volatile("" : "+v"(tcur)); }
                if (i >= 1 && NE1 + i - 1 < 16) v_consume(Sc, Pc, NE1 + i - 1, tprev);
                tprev = tcur;
                if (i >= 12) {
#pragma unroll
                    for (int q = 2 * (i - 12); q < 2 * (i - 12) + 2; ++q) {
                        pk[q] = pack2(Sc[2 * q], Sc[2 * q + 1]);
                        asm volatile("" : "+v"(pk[q]));
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (needs_mask(h + 1)) mask(h + 1, Sn, Pn);
        __builtin_amdgcn_sched_barrier(0);
        {   // D(h) with the first NE1 elements of V(h+1)
            typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
            const bf16x8 db8[2] = {__builtin_bit_cast(bf16x8, u32x4{pk[0], pk[1], pk[2], pk[3]}),
                                   __builtin_bit_cast(bf16x8, u32x4{pk[4], pk[5], pk[6], pk[7]})};
            s16x4 ring[RD][2];
#pragma unroll
            for (int i = 0; i < RD - 1; ++i) { ring[i][0] = ldd(slotD, halfD, i, 0); ring[i][1] = ldd(slotD, halfD, i, 1); }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (i + RD - 1 < 8) {
                    ring[(i + RD - 1) % RD][0] = ldd(slotD, halfD, i + RD - 1, 0);
                    ring[(i + RD - 1) % RD][1] = ldd(slotD, halfD, i + RD - 1, 1);
                }
                acc[i >> 1] = mfma32(cat4(ring[i % RD][0], ring[i % RD][1]), db8[i & 1], acc[i >> 1]);
                float tcur = 0.f;
                if (i < NE1) { tcur = v_issue(Sn, i); asm volatile("" : "+v"(tcur)); }
                if (i >= 1 && i - 1 < NE1) v_consume(Sn, Pn, i - 1, tprev);
                tprev = tcur;
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    f32x16 SA, PA, SB, PB;
    if (total > 0) {
        issue(0, 0);
        issue(1, 1);
        if constexpr (NW == 4) issue(2, 2);
        wait_vm0();
        __syncthreads();
        // M(0) and the first NE1 elements of V(0), unpipelined
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if (i & 8) PA = mfma32(ldm(lds[0], 0, i), goreg[i & 7], i == 8 ? zero16 : PA);
            else SA = mfma32(ldm(lds[0], 0, i), qreg[i & 7], i == 0 ? zero16 : SA);
        }
        if (needs_mask(0)) mask(0, SA, PA);
#pragma unroll
        for (int r = 0; r < NE1; ++r) v_consume(SA, PA, r, v_issue(SA, r));
        if constexpr (NW == 8) {
        int slot = 0;
        for (int it = 0; it < total; ++it) {
            const int slot1 = slot == 2 ? 0 : slot + 1, slot2 = slot == 0 ? 2 : slot - 1;
            if (it > 0) { wait_vm0(); __syncthreads(); }
            issue(it + 2, slot2);           // into the slot of tile it-1, which every wave has left
            stage(2 * it, SA, PA, SB, PB, lds[slot], 1, lds[slot], 0);
            stage(2 * it + 1, SB, PB, SA, PA, lds[slot1], 0, lds[slot], 1);
            slot = slot1;
        }
        } else {
        // Half h lives in slot h % 4.  Stage h reads the slots of h + 1 (M) and h (D); at the barrier in
        // front of it every wave has left stage h - 1, whose D read the slot of h - 1 = the slot of h + 3,
        // which is issued then: two stages ahead of the M that needs it.
        // (Leaving the half issued at the previous barrier in flight across the barrier, vmcnt(4) instead of
        // vmcnt(0), measured the same: the other workgroup of the CU covers the wait.)
        for (int h = 0; h < H; h += 2) {
            if (h > 0) { wait_vm0(); __syncthreads(); }
            issue(h + 3, (h + 3) & 3);
            stage(h, SA, PA, SB, PB, lds[(h + 1) & 3], 0, lds[h & 3], 0);
            wait_vm0();
            __syncthreads();
            issue(h + 4, h & 3);
            stage(h + 1, SB, PB, SA, PA, lds[(h + 2) & 3], 0, lds[(h + 1) & 3], 0);
        }
        }
    }

    // D = sum_s P dP equals rowsum(dO * O) exactly, but does not inherit the bf16 rounding of O.
    // Publish it for the dkdv pass (this workgroup owns these rows of D, so overwriting is safe).
    dsum = pair_sum(dsum);
    const bool store = valid && !(a.resp_only && t < Lp);
    if (store && hh == 0) a.D[(int64_t)head * T_total + gd.tok_base + t] = dsum;
    // rows that see at most EDGE_LEN keys are written by the edge kernel (fp32 dS): not stored here
    const bool short_row = (t < Lp ? 0 : Lp) + t - st + 1 <= EDGE_LEN;
    if (store && !short_row) {
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
__shared__ __attribute__((aligned(1024))) char dkdv_ldsKV[2][128 * 256];       // [K | V] of the 128 keys
__shared__ __attribute__((aligned(1024))) char dkdv_lds[2][2 * TILE_BYTES];    // [buffer][Q | dO]
__shared__ __attribute__((aligned(256))) float dkdv_ldsLD[2][2][64];           // [buffer][L2 | D][row]

__device__ __forceinline__ void dkdv_body(const BwdArgs& a, const TileDesc td, const int kvh, const int hr_only) {
    const int ti = td.ti;
    constexpr int BNK = 128, BQ = 64;
    constexpr int RD = 3;      // LDS operand ring depth (prefetch distance RD - 1 MFMAs)
    const int s0 = ti * BNK;
    GroupDesc gd;
    gd.tok_base = td.tok_base; gd.Lp = td.Lp; gd.Tg = td.Tg; gd.G = 0; gd.roff = nullptr;
    const int Lp = gd.Lp, Tg = gd.Tg;
    const int64_t T_total = a.tab[1];

    const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), l = tid & 63;
    const int c = l & 31, hh = l >> 5, j = l & 15, c16 = (l >> 4) & 1;
    const int kb = w & 3, qh = w >> 2;

    // this lane's key (a column of S) and the rows [s, e_s) that may see it
    const int s = s0 + 32 * kb + c;
    const bool valid = s < Tg;
    const int ws0 = s0 + 32 * kb;                      // wave's first key
    const bool wave_valid = ws0 < Tg;
    const int ws1 = min(ws0 + 31, Tg - 1);             // wave's last valid key
    const int s1 = min(s0 + BNK, Tg);
    // rows [s, e_s) see this lane's key; row_end: where the rows that see any key of the tile end (the
    // group's end if the tile holds a prompt key, else the end of its last key's response)
    const int e_s = valid ? a.sched.row_hi[gd.tok_base + s] : 0;
    const int row_end = __builtin_amdgcn_readfirstlane(s0 < Lp ? Tg : a.sched.row_hi[gd.tok_base + s1 - 1]);
    // smallest / largest row bound e_s over the wave's keys (prompt keys: Tg; response keys: the
    // end of their response, non-decreasing in s); lanes 0..31 hold the wave's keys in order
    const int e_min = !wave_valid ? 0 : (ws1 < Lp ? Tg : __builtin_amdgcn_readlane(e_s, max(ws0, Lp) - ws0));
    const int e_max = !wave_valid ? 0 : (ws0 < Lp ? Tg : __builtin_amdgcn_readlane(e_s, ws1 - ws0));

    // with only response rows contributing, the rows start at the end of the prompt
    const int row_lo = a.resp_only ? Lp : 0;
    const int s_lo = max(s, row_lo);                   // first row that contributes to this lane's key
    const int qt0 = max(s0, row_lo) / BQ, qt1 = (row_end + BQ - 1) / BQ;
    const int rep_all = a.Hq / a.Hkv;
    const int rep = a.head_split ? 1 : rep_all;        // q heads this workgroup walks
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
            async_copy16(src, &dkdv_ldsKV[ci >> 5][(ci & 31) * 1024]);
        }
    }
    // Row tiles are walked from the LAST one down to the workgroup's own keys: workgroups that
    // start together (they share a kv head and an XCD) then stream the same Q/dO tiles at the
    // same time, so all but the first read of a tile hit that XCD's L2.
    // The q heads of the kv head are the inner loop, for the same reason.
    // Step `it` = (row tile qt1 - 1 - it / rep, q head it % rep).  Its Q/dO tile is copied
    // asynchronously into buffer it & 1: wave w copies chunks 2w, 2w+1 (4 rows each) of Q and of
    // dO, from a scalar tile base plus a constant per-lane offset.  (The copies wait on HBM, and a
    // wave that queues more than a few of them stalls at issue, so all eight waves share them.)
    // Rows past the group's end re-read its last row; they are masked (t < e_s <= Tg fails).
    const unsigned qstride_b = (unsigned)(q_stride * 2);
    unsigned voff[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int row = 4 * (2 * w + u) + (l >> 4);
        voff[u] = row * qstride_b + (((l & 15) ^ swz(row)) << 4);
    }
    auto sgpr64 = [](const void* p) -> uint64_t {
        const uint64_t b = (uint64_t)(uintptr_t)p;
        return ((uint64_t)(unsigned)__builtin_amdgcn_readfirstlane((int)(b >> 32)) << 32) |
               (uint64_t)(unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)b);
    };
    auto lds_u32 = [](const void* p) -> unsigned {
        return __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(__attribute__((address_space(3))) const char*)p);
    };
    // first q head of this workgroup, token 0 of the group
    const int head0 = kvh * rep_all + hr_only;          // first q head this workgroup walks
    const uint64_t qbase_s = sgpr64(a.q + ((int64_t)gd.tok_base * a.Hq + head0) * 128);
    const uint64_t gbase_s = sgpr64(a.d_o + ((int64_t)gd.tok_base * a.Hq + head0) * 128);
    const unsigned m0buf[2] = {lds_u32(dkdv_lds[0]) + 2048u * w, lds_u32(dkdv_lds[1]) + 2048u * w};
    const unsigned tile_bytes = BQ * qstride_b;
    auto issue_tile = [&](int qt, int hr, int buf) {
        const uint64_t off = (uint64_t)(unsigned)qt * tile_bytes + (unsigned)hr * 256u;
        const unsigned m0 = m0buf[buf];
        if (qt * BQ + BQ <= Tg) {
#pragma unroll
            for (int u = 0; u < 2; ++u) async_copy16_sm(qbase_s + off, voff[u], m0 + 1024u * u);
#pragma unroll
            for (int u = 0; u < 2; ++u) async_copy16_sm(gbase_s + off, voff[u], m0 + TILE_BYTES + 1024u * u);
        } else {
            const int last = Tg - 1 - qt * BQ;
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int row = 4 * (2 * w + u) + (l >> 4);
                const unsigned vo = min(row, last) * qstride_b + (((l & 15) ^ swz(row)) << 4);
                async_copy16_sm(qbase_s + off, vo, m0 + 1024u * u);
                async_copy16_sm(gbase_s + off, vo, m0 + TILE_BYTES + 1024u * u);
            }
        }
        if (w < 2) {        // wave 0: scaled LSE of the 64 rows, wave 1: D (the first wave of a SIMD has slack)
            const int head = head0 + hr;
            const int t = min(qt * BQ + l, Tg - 1);
            const float* src = (w == 0 ? a.L2 : a.D) + (int64_t)head * T_total + gd.tok_base + t;
            async_copy4(src, reinterpret_cast<char*>(&dkdv_ldsLD[buf][w][0]));
        }
    };

    f32x16 dkacc[4], dvacc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) { dkacc[db][r] = 0.f; dvacc[db][r] = 0.f; }
    const float cs = a.c;
    const char* ldsK = dkdv_ldsKV[0];
    const char* ldsV = dkdv_ldsKV[1];
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

    // Within a step the vector work is folded under the MFMAs: the exponentials of the first 8
    // rows run under the dP MFMAs (S is complete by then), those of the last 8 rows under the
    // first half of the dV/dK MFMAs (which only need the first 8 rows of P and dS).  Masking is
    // applied to S beforehand (score -inf gives P = 0 and dS = 0).
    // Rows that see only a few keys carry weights P of order one, and a key's dK / dV can be made up almost
    // entirely of a handful of such terms, whose bf16 roundings of P and dS then do not average out.  The
    // steps that hold such rows (the first EDGE_LEN rows of a prompt; under a shorter prompt, conservatively,
    // every step with response rows) are therefore swept a second time after the main sweep, with P and dS
    // replaced by what their rounding dropped, P - bf16(P) and dS - bf16(dS) (rounded to bf16 in turn): the
    // two sweeps together carry P and dS into dV and dK to about 2^-17.  The second sweep is the same code
    // with another packing function, outside the main loop, so it costs that loop neither registers nor time.
    auto sweep = [&](auto lo_tag, const int q_hi, const int q_lo) {      // row tiles q_hi - 1 down to q_lo
    constexpr bool LO = decltype(lo_tag)::value;
    auto pack2 = [&](float x, float y) -> unsigned {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        bf16x2 v = {(__bf16)x, (__bf16)y};
        if (LO) v = bf16x2{(__bf16)(x - (float)v[0]), (__bf16)(y - (float)v[1])};
        return __builtin_bit_cast(unsigned, v);
    };
    const int n_steps = max(q_hi - q_lo, 0) * rep;
    int qt = q_hi - 1, hr = 0;                // step 0
    int qt_n = qt, hr_n = 1;                  // step 1
    if (hr_n == rep) { hr_n = 0; --qt_n; }
    if (n_steps > 0) issue_tile(qt, hr, 0);
    for (int it = 0; it < n_steps; ++it) {
        const int buf = it & 1;
        wait_vm0();
        __syncthreads();
        const char* ldsQ = dkdv_lds[buf];
        const char* ldsG = dkdv_lds[buf] + TILE_BYTES;
        const float* ldsL = dkdv_ldsLD[buf][0];
        const float* ldsD = dkdv_ldsLD[buf][1];
        const int r0 = qt * BQ + 32 * qh;              // this wave's 32 rows
        const int qt_n_issue = qt_n, hr_n_issue = hr_n;
        qt = qt_n; hr = hr_n;
        if (++hr_n == rep) { hr_n = 0; --qt_n; }
        // no row of this wave's half sees any key of this wave
        const bool skip = !wave_valid || r0 + 31 < max(ws0, row_lo) || r0 >= e_max ||
                          (LO && !(r0 < min(Lp, EDGE_LEN) || (Lp < EDGE_LEN && r0 + 31 >= Lp)));   // or: no short row here

        // The LDS operands of the step's 32 MFMAs pass through one pair of rings, read RD - 1 MFMAs ahead
        // without a break between the four products (a product that primed rings of its own would start with
        // an exposed LDS round trip).  Slice i: 0..7 S = Q K^T, 8..15 dP = dO V^T, 16..23 and 24..31 the dV / dK
        // updates for the first and the last 16 rows of the block (A operand only: P and dS are in registers).
        auto ldt = [&](int mm, int i, int part) {       // dV for even i, dK for odd i; db = i / 2
            const int col4 = 32 * (i >> 1) + 16 * c16 + 4 * (j & 3);
            const int row4 = 32 * qh + 16 * mm + 4 * hh + (j >> 2);
            return lds_read_tr4((i & 1) ? ldsQ : ldsG, row4 + 8 * part, col4);
        };
        auto fetchA = [&](int i) -> bf16x8 {
            if (i < 8) return lds_read_row8(ldsQ, 32 * qh + c, 2 * i + hh);
            if (i < 16) return lds_read_row8(ldsG, 32 * qh + c, 2 * (i - 8) + hh);
            return cat4(ldt((i - 16) >> 3, i & 7, 0), ldt((i - 16) >> 3, i & 7, 1));
        };
        auto fetchB = [&](int i) -> bf16x8 {
            return lds_read_row8(i < 8 ? ldsK : ldsV, 32 * kb + c, 2 * (i & 7) + hh);
        };
        bf16x8 ra[RD], rb[RD];
        auto advance = [&](int i) {                      // fetch the operands of slice i + RD - 1
            const int n = i + RD - 1;
            if (n < 32) ra[n % RD] = fetchA(n);
            if (n < 16) rb[n % RD] = fetchB(n);
        };
        // the first operands are fetched ahead of the issue of the next tile's copies, which every wave takes
        // part in whether it has work in this step or not
        if (!skip) {
#pragma unroll
            for (int i = 0; i < RD - 1; ++i) { ra[i] = fetchA(i); rb[i] = fetchB(i); }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (it + 1 < n_steps) issue_tile(qt_n_issue, hr_n_issue, buf ^ 1);
        if (skip) continue;
        f32x16 sacc, pacc;
#pragma unroll
        for (int i = 0; i < 8; ++i) {       // S = Q K^T
            advance(i);
            sacc = mfma32(ra[i % RD], rb[i % RD], i == 0 ? zero16 : sacc);
            __builtin_amdgcn_sched_barrier(0);
        }
        // every row of the half sees every key of the wave
        const bool full = r0 >= max(ws1, row_lo) && ws0 + 31 < Tg && r0 + 32 <= e_min;
        if (!full) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int t = r0 + 8 * (r >> 2) + 4 * hh + (r & 3);
                sacc[r] = (t >= s_lo && t < e_s) ? sacc[r] : -INFINITY;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        float Lr[16], Dr[16];
        {   // dP = dO V^T, with the exponentials of rows 0..7 of the block
#pragma unroll
            for (int gq = 0; gq < 2; ++gq) {
                const f32x4 L4 = *reinterpret_cast<const f32x4*>(&ldsL[32 * qh + 8 * gq + 4 * hh]);
#pragma unroll
                for (int e = 0; e < 4; ++e) Lr[4 * gq + e] = L4[e];
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                advance(8 + i);
                if (i == 2 || i == 3) {         // D of rows 0..7, L of rows 8..15
                    const f32x4 D4 = *reinterpret_cast<const f32x4*>(&ldsD[32 * qh + 8 * (i - 2) + 4 * hh]);
                    const f32x4 L4 = *reinterpret_cast<const f32x4*>(&ldsL[32 * qh + 8 * i + 4 * hh]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) { Dr[4 * (i - 2) + e] = D4[e]; Lr[4 * i + e] = L4[e]; }
                }
                pacc = mfma32(ra[(8 + i) % RD], rb[(8 + i) % RD], i == 0 ? zero16 : pacc);
                sacc[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[i], cs, -Lr[i]));      // P
                asm volatile("" : "+v"(sacc[i]));
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        unsigned pp[8], dd[8];       // packed bf16 pairs of P and dS: [4 * mm + r / 2]
#pragma unroll
        for (int r = 0; r < 8; ++r) pacc[r] = sacc[r] * (pacc[r] - Dr[r]);               // dS
#pragma unroll
        for (int q = 0; q < 4; ++q) { pp[q] = pack2(sacc[2 * q], sacc[2 * q + 1]); dd[q] = pack2(pacc[2 * q], pacc[2 * q + 1]); }
        __builtin_amdgcn_sched_barrier(0);
        // dV^T += dO^T P, dK^T += Q^T dS
        {   // first 16 rows of the block (mm = 0), with the exponentials and dS of rows 8..15
            const bf16x8 p8 = __builtin_bit_cast(bf16x8, u32x4{pp[0], pp[1], pp[2], pp[3]});
            const bf16x8 d8 = __builtin_bit_cast(bf16x8, u32x4{dd[0], dd[1], dd[2], dd[3]});
#pragma unroll
            for (int gq = 2; gq < 4; ++gq) {
                const f32x4 D4 = *reinterpret_cast<const f32x4*>(&ldsD[32 * qh + 8 * gq + 4 * hh]);
#pragma unroll
                for (int e = 0; e < 4; ++e) Dr[4 * gq + e] = D4[e];
            }
            __builtin_amdgcn_sched_barrier(0);
            float tprev = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                advance(16 + i);
                const bf16x8 A = ra[(16 + i) % RD];
                if (i & 1) dkacc[i >> 1] = mfma32(A, d8, dkacc[i >> 1]);
                else dvacc[i >> 1] = mfma32(A, p8, dvacc[i >> 1]);
                float tcur = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[8 + i], cs, -Lr[8 + i]));
                asm volatile("" : "+v"(tcur));
                if (i >= 1) {
                    sacc[8 + i - 1] = tprev;
                    pacc[8 + i - 1] = tprev * (pacc[8 + i - 1] - Dr[8 + i - 1]);
                    asm volatile("" : "+v"(pacc[8 + i - 1]));
                }
                tprev = tcur;
                __builtin_amdgcn_sched_barrier(0);
            }
            sacc[15] = tprev;
            pacc[15] = tprev * (pacc[15] - Dr[15]);
        }
#pragma unroll
        for (int q = 4; q < 8; ++q) { pp[q] = pack2(sacc[2 * q], sacc[2 * q + 1]); dd[q] = pack2(pacc[2 * q], pacc[2 * q + 1]); }
        __builtin_amdgcn_sched_barrier(0);
        {   // last 16 rows of the block (mm = 1)
            const bf16x8 p8 = __builtin_bit_cast(bf16x8, u32x4{pp[4], pp[5], pp[6], pp[7]});
            const bf16x8 d8 = __builtin_bit_cast(bf16x8, u32x4{dd[4], dd[5], dd[6], dd[7]});
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                advance(24 + i);
                const bf16x8 A = ra[(24 + i) % RD];
                if (i & 1) dkacc[i >> 1] = mfma32(A, d8, dkacc[i >> 1]);
                else dvacc[i >> 1] = mfma32(A, p8, dvacc[i >> 1]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    };
    sweep(std::false_type{}, qt1, qt0);
    {   // the steps that can hold short rows: row tile 0 under a prompt of at least EDGE_LEN tokens, else all
        const int f_hi = Lp >= EDGE_LEN ? min(qt1, 1) : qt1;
        if (f_hi > qt0) {
            __syncthreads();                       // every wave has left the main sweep's last buffer
            sweep(std::true_type{}, f_hi, qt0);
        }
    }

    // add the two row halves: waves 4..7 park their partial sums in LDS (the Q/dO buffers,
    // 16 KB per wave), waves 0..3 add them and write the result.  dK first, then dV.
    float* xch = reinterpret_cast<float*>(&dkdv_lds[0][0]) + (size_t)kb * 4096 + l * 4;
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
                    if (a.head_split) {      // fp32 partial sum of this q head; scaled and rounded by the reduce kernel
                        float* part = a.partial + ((int64_t)pass * rep_all + hr_only) * T_total * a.Hkv * 128;
                        const f32x4 z = {acc[db][4 * gq] + y[0], acc[db][4 * gq + 1] + y[1], acc[db][4 * gq + 2] + y[2],
                                         acc[db][4 * gq + 3] + y[3]};
                        *reinterpret_cast<f32x4*>(part + orow + 32 * db + 8 * gq) = z;
                        continue;
                    }
                    bf16x4 x;
                    bf16x4 old = {0, 0, 0, 0};
                    if (a.accumulate) old = *reinterpret_cast<const bf16x4*>(out + orow + 32 * db + 8 * gq);
#pragma unroll
                    for (int e = 0; e < 4; ++e) x[e] = (__bf16)((acc[db][4 * gq + e] + y[e]) * mul + (float)old[e]);
                    *reinterpret_cast<bf16x4*>(out + orow + 32 * db + 8 * gq) = x;
                }
        }
    }
}

__global__ __launch_bounds__(512) void bwd_dkdv_kernel(BwdArgs a) {
    int tile, kvh, hr_only = 0;
    if (a.head_split) {
        int head;
        if (!decode_item(blockIdx.x, a.n_tiles, a.Hq, a.Hkv, tile, head)) return;
        kvh = head / (a.Hq / a.Hkv);
        hr_only = head % (a.Hq / a.Hkv);
    } else if (!decode_item(blockIdx.x, a.n_tiles, a.Hkv, a.Hkv, tile, kvh)) return;
    // key tiles in ascending order: the first prompt tile is seen by every row (most work)
    dkdv_body(a, a.sched.tiles128[tile], kvh, hr_only);
}

// Second stage of the head-split dkdv pass: dk = scale * sum_hr partial[0][hr], dv = sum_hr
// partial[1][hr], summed in a fixed order (bitwise repeatable), rounded once, optionally added
// to what the outputs hold.  One thread per 4 consecutive elements.
__global__ __launch_bounds__(256) void dkdv_reduce_kernel(const float* __restrict__ partial, __bf16* __restrict__ dk,
                                                          __bf16* __restrict__ dv, int64_t n4, int rep, float scale,
                                                          int accumulate) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n4) return;
    const int64_t plane = n4 * 4;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int hr = 0; hr < rep; ++hr) {
            const f32x4 x = *reinterpret_cast<const f32x4*>(partial + ((int64_t)pass * rep + hr) * plane + 4 * i);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] += x[e];
        }
        __bf16* out = (pass == 0 ? dk : dv) + 4 * i;
        const float mul = pass == 0 ? scale : 1.0f;
        bf16x4 old = {0, 0, 0, 0};
        if (accumulate) old = *reinterpret_cast<const bf16x4*>(out);
        bf16x4 r;
#pragma unroll
        for (int e = 0; e < 4; ++e) r[e] = (__bf16)(acc[e] * mul + (float)old[e]);
        *reinterpret_cast<bf16x4*>(out) = r;
    }
}

}  // namespace

hipError_t launch_bwd_bf16(const Problem& p, hipStream_t s) {
    hipError_t e = hipSuccess;
    // A call that runs both the rowsum and the dq stage folds the first into the second (the dq pass has
    // the dO rows in registers anyway): one pass over o and dO less.  Not in response-rows mode, where the
    // dq pass skips the prompt's tiles and the dkdv pass still needs finite planes for every row it loads,
    // and not for head counts that the layout of rowsum_bf16_kernel (whose arithmetic the fold repeats) does not take.
    const bool fused = (p.stages & STAGE_ROWSUM) && (p.stages & STAGE_DQ) && !p.resp_only && rowsum_fast_path(p);
    if ((p.stages & STAGE_ROWSUM) && !fused) {
        e = launch_rowsum(p, false, s);
        if (e != hipSuccess) return e;
    }
    BwdArgs a{};
    a.fused_rowsum = fused; a.o = (const __bf16*)p.o; a.o_lo = (const __bf16*)p.o_lo; a.lo_flag = p.o_lo_flag;
    a.q = (const __bf16*)p.q; a.k = (const __bf16*)p.k; a.v = (const __bf16*)p.v; a.d_o = (const __bf16*)p.d_o;
    a.lse = p.lse; a.D = p.Dbuf; a.L2 = p.Dbuf + (int64_t)p.Hq * p.total_tokens;
    a.dq = (__bf16*)p.dq; a.dk = (__bf16*)p.dk; a.dv = (__bf16*)p.dv;
    a.tab = p.tab; a.sched = p.sched; a.n_groups = p.n_groups; a.Hq = p.Hq; a.Hkv = p.Hkv; a.scale = p.scale; a.c = p.scale * LOG2E;
    a.resp_only = p.resp_only; a.accumulate = p.accumulate;
    if (p.stages & STAGE_DQ) {
        // short key loops: the 128-row shape, two workgroups per CU (the forward's rule, see bwd_dq_kernel)
        const bool small = use_small_shape(p);
        a.n_tiles = count_tiles(p, small ? 128 : 256);
        const int grid = grid_for_items(a.n_tiles, p.Hq, p.Hkv);
        if (small) hipLaunchKernelGGL(bwd_dq_kernel<4>, dim3(grid), dim3(256), 0, s, a);
        else hipLaunchKernelGGL(bwd_dq_kernel<8>, dim3(grid), dim3(512), 0, s, a);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        e = launch_short_rows(p, true, s);
        if (e != hipSuccess) return e;
    }
    if (p.stages & STAGE_DKDV) {
        a.n_tiles = count_tiles(p, 128);
        a.head_split = p.dkdv_partial != nullptr;
        a.partial = p.dkdv_partial;
        if (a.head_split) {
            const int grid = grid_for_items(a.n_tiles, p.Hq, p.Hkv);
            hipLaunchKernelGGL(bwd_dkdv_kernel, dim3(grid), dim3(512), 0, s, a);
            const int64_t n4 = p.total_tokens * p.Hkv * 32;
            hipLaunchKernelGGL(dkdv_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s, a.partial, a.dk, a.dv,
                               n4, p.Hq / p.Hkv, p.scale, a.accumulate);
        } else {
            const int grid = grid_for_items(a.n_tiles, p.Hkv, p.Hkv);
            hipLaunchKernelGGL(bwd_dkdv_kernel, dim3(grid), dim3(512), 0, s, a);
        }
        e = hipGetLastError();
    }
    return e;
}

}  // namespace sp
