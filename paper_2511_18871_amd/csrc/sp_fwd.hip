// Forward shared-prompt attention, bf16 MFMA path (gfx950).
//
// One workgroup owns a tile of 256 consecutive packed query rows of one group and one
// q head; wave w (of 8) owns 32 of those rows.  Keys/values stream through LDS in tiles of
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
#include <type_traits>

namespace sp {
namespace {

constexpr int BN = 64;                 // keys per LDS tile
constexpr float P_LIMIT = 16384.0f;     // bound on a lane's per-tile sum of exponentials (2^14)
constexpr int TILE_BYTES = BN * 256;   // 64 rows x 128 bf16
constexpr float M_NONE = -1.0e30f;     // reference point of a row that has not seen a key yet (finite on purpose)

struct FwdArgs {
    // one entry per tensor set; the sets share the packing, the schedule and the launch
    const __bf16* q[MAX_SETS]; const __bf16* k[MAX_SETS]; const __bf16* v[MAX_SETS];
    __bf16* o[MAX_SETS]; float* lse[MAX_SETS];
    int blocks_per_set;
    const int* tab;
    Schedule sched; // tile descriptors and per-token segment bounds, written by the schedule kernel of the call
    int n_tiles, n_groups, Hq, Hkv;
    float c;        // softmax_scale * log2(e)
    int naive;
    int resp_only;  // compute and write response rows only
    __bf16* o_lo;   // optional (single-set launches): o_fp32 - bf16(o), rounded to bf16, same layout as o
};

// ------------------------------------------------------------------------------------
// Hand-scheduled software-pipelined forward.  Step j of a wave holds the MFMAs of two tiles and
// the vector-ALU work of a third:
//   O^T += V(j-1)^T P(j-1)^T  (16 MFMAs),  S(j+1) = K(j+1) Q^T  (16 MFMAs),
//   P(j) = exp2(S(j) c - m c), its row sums and its bf16 packing  (32 scores per lane).
// The step is written as 32 slices of {LDS operand read for the MFMA two slices ahead, one
// MFMA, the vector work of one score}, fenced so the compiler keeps that order: while MFMAs
// stream, a SIMD takes about five other vector instructions per MFMA for free, which is what a
// slice holds.  So that the exponentials can be spread this evenly they are taken against the
// reference point m the row had before the tile (see `step`).  Two steps run per workgroup
// barrier; the K and V tiles of the following two steps are copied into LDS meanwhile.
// ------------------------------------------------------------------------------------
//
// Two shapes of workgroup.  NW = 8: 256 rows, four K and four V buffers (128 KB of LDS), one workgroup
// per CU: the shape for long key loops.  NW = 4: 128 rows, two K and two V buffers (64 KB), one step
// per barrier, TWO workgroups per CU: each workgroup's fixed costs (table lookups, first loads,
// epilogue, the gap before the next dispatch) then overlap with the other's key loop, which is what
// batches of short groups need, where a workgroup runs only a handful of steps.
// NAIVE = the measurement baseline (every tile at or below the packed diagonal, mask applied element by
// element): a separate instantiation, so that it shows under its own name in kernel traces and its
// branches cost the product kernel nothing.
template <int NW, bool NAIVE>
__global__ __launch_bounds__(NW * 64, 2) void fwd_kernel(FwdArgs a) {      // two waves per SIMD in either shape
    constexpr int BM = 32 * NW;
    constexpr int NB = NW == 8 ? 4 : 2;            // K buffers = V buffers
    constexpr int RD = 3;      // LDS operand ring depth (prefetch distance RD - 1 MFMAs)
    __shared__ __attribute__((aligned(1024))) char ldsKb[NB][TILE_BYTES];      // K tile t lives in ldsKb[t % NB]
    __shared__ __attribute__((aligned(1024))) char ldsVb[NB][TILE_BYTES];      // V tile t in ldsVb[t % NB]

    // blocks are dealt set-major; blocks_per_set is a multiple of 8, so the block -> XCD mapping
    // of a set does not depend on how many sets the launch carries
    const int set = blockIdx.x / a.blocks_per_set;
    const __bf16* const aq = a.q[set]; const __bf16* const ak = a.k[set]; const __bf16* const av = a.v[set];
    __bf16* const ao = a.o[set]; float* const alse = a.lse[set];
    int tile, head;
    if (!decode_item(blockIdx.x - set * a.blocks_per_set, a.n_tiles, a.Hq, a.Hkv, tile, head)) return;
    // the tile's descriptor: one 32-byte load instead of a bisection over the groups and the group's entry
    const TileDesc td = (BM == 256 ? a.sched.tiles256 : a.sched.tiles128)[tile];
    const int ti = td.ti;
    GroupDesc gd;
    gd.tok_base = td.tok_base; gd.Lp = td.Lp; gd.Tg = td.Tg; gd.G = 0; gd.roff = nullptr;
    const int Lp = gd.Lp, Tg = gd.Tg;
    const int t0 = ((Tg + BM - 1) / BM - 1 - ti) * BM;   // a group's last tile first: it carries the most work
    const int T_total = a.tab[1];
    if (a.resp_only && t0 + BM <= Lp) return;      // a tile of prompt rows only

    const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), l = tid & 63;
    const int c = l & 31, hh = l >> 5, j16 = l & 15, c16 = (l >> 4) & 1;

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

    bf16x8 qreg[8];
    {
        // rows past the end of the group read the group's last row instead: every score of such a
        // row is masked and nothing of it is stored, and without a select on the loaded value the
        // wait for these loads moves down to the first MFMA, behind the issue of the tile copies
        const __bf16* qp = aq + ((int64_t)(gd.tok_base + min(t, Tg - 1)) * a.Hq + head) * 128 + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
    }

    const int t1 = min(t0 + BM, Tg);
    int n1, k2b, k2e;
    if (NAIVE) {
        n1 = (t1 + BN - 1) / BN; k2b = k2e = n1;
    } else {
        n1 = (min(Lp, t1) + BN - 1) / BN;
        k2b = k2e = n1;
        if (t1 > Lp) {
            k2b = max(n1, b2 / BN);
            k2e = (t1 + BN - 1) / BN;
        }
    }
    const int total = n1 + (k2e - k2b);
    auto tile_at = [&](int it) { return it < n1 ? it : k2b + (it - n1); };

    const int kvh = head / (a.Hq / a.Hkv);
    const int64_t kv_stride = (int64_t)a.Hkv * 128;
    const __bf16* kbase = ak + ((int64_t)gd.tok_base * a.Hkv + kvh) * 128;
    const __bf16* vbase = av + ((int64_t)gd.tok_base * a.Hkv + kvh) * 128;

    // Tile copy global -> LDS.  The first wave of each SIMD (w < 4) is served first by the
    // instruction arbiter and reaches the workgroup barrier well ahead of its partner, so those
    // four waves issue all the copies: wave w copies chunks 4w .. 4w+3 (4 rows each) of a 64-row
    // tile.  The per-lane byte offset inside a tile is constant; only the scalar tile base moves.
    // The tile that crosses the end of the group re-reads the group's last row for the rows past it.
    const unsigned stride_b = (unsigned)(kv_stride * 2);
    const bool copier = w < 4;
    unsigned voff[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int row = 4 * (4 * (w & 3) + u) + (l >> 4);
        voff[u] = row * stride_b + (((l & 15) ^ swz(row)) << 4);
    }
    auto sgpr64 = [](const void* p) -> uint64_t {       // a wave-uniform pointer, kept in scalar registers
        const uint64_t b = (uint64_t)(uintptr_t)p;
        return ((uint64_t)(unsigned)__builtin_amdgcn_readfirstlane((int)(b >> 32)) << 32) |
               (uint64_t)(unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)b);
    };
    const uint64_t kbase_s = sgpr64(kbase), vbase_s = sgpr64(vbase);
    const unsigned tile_bytes = BN * stride_b;
    auto lds_u32 = [](char* p) -> unsigned {
        return __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)p);
    };
    const unsigned chunk0 = 4096u * (w & 3);
    unsigned m0K[NB], m0V[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) { m0K[b] = lds_u32(ldsKb[b]) + chunk0; m0V[b] = lds_u32(ldsVb[b]) + chunk0; }
    auto issue = [&](uint64_t base_s, unsigned m0dst, int it) {
        if (!copier || it >= total) return;
        const int kt = tile_at(it);
        const uint64_t tb = base_s + (uint64_t)(unsigned)kt * tile_bytes;
        if (kt * BN + BN <= Tg) {
#pragma unroll
            for (int u = 0; u < 4; ++u) async_copy16_sm(tb, voff[u], m0dst + 1024u * u);
        } else {
            const int last = Tg - 1 - kt * BN;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int row = 4 * (4 * (w & 3) + u) + (l >> 4);
                const unsigned vo = min(row, last) * stride_b + (((l & 15) ^ swz(row)) << 4);
                async_copy16_sm(tb, vo, m0dst + 1024u * u);
            }
        }
    };
    // true when some (row, key) pair of this wave in tile `it` is masked; tiles past the end
    // of the key range (the pad step of an odd-length loop) are masked entirely
    // the first n_full tiles (whole prompt tiles at or below the wave's first row) never need it
    const int n_full = (!wave_valid || NAIVE) ? 0 : __builtin_amdgcn_readfirstlane(min(min(Lp, tw0 + 1) / BN, n1));
    auto needs_mask = [&](int it) -> bool {
        if (it < n_full) return false;
        if (it >= total || !wave_valid || NAIVE) return true;
        const int s0 = tile_at(it) * BN;
        return !((s0 + BN - 1 <= tw0) && (s0 + BN <= Lp || s0 >= st_last));
    };

    f32x16 oacc[4], sA[2], sB[2];
    unsigned pbA[16], pbB[16]; // P of a tile as packed bf16 pairs, [8*kb + r/2]; the two alternate from step to step
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) { pbA[i] = 0u; pbB[i] = 0u; }
    float m = -INFINITY, lsum = 0.f, lsr = 0.f;
    const float cs = a.c;
    const f32x16 zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

    // operand fetchers, all indices compile-time
    auto ldK = [&](const char* ldsK, int i) -> bf16x8 {         // MFMA i of QK: kb = i / 8, ks = i % 8
        return lds_read_row8(ldsK, 32 * (i >> 3) + c, 2 * (i & 7) + hh);
    };
    auto ldV = [&](const char* ldsV, int i, int half) -> s16x4 { // MFMA i of PV: kb = i / 8, mm = (i / 4) % 2, db = i % 4
        const int col4 = 32 * (i & 3) + 16 * c16 + 4 * (j16 & 3);
        const int row4 = 32 * (i >> 3) + 16 * ((i >> 2) & 1) + 4 * hh + (j16 >> 2) + 8 * half;
        return lds_read_tr4(ldsV, row4, col4);
    };
    auto pbop = [&](const unsigned (&pbw)[16], int kb, int mm) -> bf16x8 {
        typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
        u32x4 x = {pbw[8 * kb + 4 * mm], pbw[8 * kb + 4 * mm + 1], pbw[8 * kb + 4 * mm + 2], pbw[8 * kb + 4 * mm + 3]};
        return __builtin_bit_cast(bf16x8, x);
    };
    auto sum2 = [&](unsigned packed, float acc) -> float {       // acc + both bf16 halves of `packed`
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        const bf16x2 one = {(__bf16)1.0f, (__bf16)1.0f};
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, packed), one, acc, false);
    };
    auto pack2 = [&](float x, float y) -> unsigned {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        bf16x2 v = {(__bf16)x, (__bf16)y};
        return __builtin_bit_cast(unsigned, v);
    };

    // the first S = K Q^T, ahead of the pipeline
    auto qk_plain = [&](const char* ldsK, f32x16 (&S)[2]) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
            S[i >> 3] = mfma32(ldK(ldsK, i), qreg[i & 7], (i & 7) == 0 ? zero16 : S[i >> 3]);
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

    // one pipeline step for tile j (R = j & 3 selects the LDS buffers): Scur holds S(j), Snext receives S(j+1).
    // Every wave runs every step: tiles it cannot see are handled by the mask (P = 0), the
    // first step multiplies the zero P against a zero-filled V buffer, and the last step's
    // S(j+1) is computed from a stale K buffer and never used.
    //
    // The exponentials of S(j) are taken against the reference point m that the row had BEFORE
    // this tile, so they do not wait for the tile's row maximum and can be spread evenly, one
    // element per MFMA slice, over the 32 MFMAs of the step (16 of O += V(j-1) P(j-1), then 16
    // of S(j+1) = K(j+1) Q^T).  The softmax is shift-invariant, so any finite reference gives
    // the same O and LSE; what has to hold is that the exponentials stay in range.  That is
    // checked after the fact: if a lane's 32 exponentials sum to more than P_LIMIT = 2^14 (or
    // to inf/NaN), the wave takes the exact row maximum as the new reference, rescales O and
    // the row sum, and recomputes this tile's P -- a rare path, taken a few times per row.
    // The LDS operands of the step's 32 MFMAs pass through one ring of RD registers that is read RD - 1
    // MFMAs ahead without a break between the two products: a product that primed its own ring would
    // start with an exposed LDS round trip.  Between the two steps of a barrier interval the ring is
    // carried over as well (BRIDGE: the last slices fetch the first operands of the next step, whose V
    // tile is resident; SECOND: the step finds them there): only the first step behind a barrier primes.
    // (Priming right behind the barrier, ahead of the issue of the tile copies, measured the same.)
    bf16x8 ring[RD];
    auto step = [&](int j, auto par_tag, auto second_tag, auto bridge_tag, f32x16 (&Scur)[2], f32x16 (&Snext)[2],
                    const unsigned (&pbw)[16], unsigned (&pnew)[16]) {
        constexpr int R = decltype(par_tag)::value;
        constexpr bool SECOND = decltype(second_tag)::value, BRIDGE = decltype(bridge_tag)::value;
        constexpr int OFF = SECOND ? 32 % RD : 0;     // ring position of this step's first operand
        const char* ldsV = ldsVb[(R + NB - 1) % NB];  // V(j-1)
        const char* ldsK = ldsKb[(R + 1) % NB];       // K(j+1)
        const char* ldsVn = ldsVb[R % NB];            // V(j), the next step's
        if (needs_mask(j)) mask(j, Scur);
        __builtin_amdgcn_sched_barrier(0);
        const float mc = m * cs;
        float tsum = 0.f;          // this lane's half of the tile's row sum
        float tsr = 0.f;           // the same sum over the bf16-rounded exponentials (what the MFMA multiplies V by)
        float pe[32];
        // vector-ALU slice e: exponential of element e; the sum and the bf16 packing consume
        // elements issued in earlier slices, so nothing waits on a transcendental just issued
        auto valu = [&](int e) {
            pe[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(Scur[e >> 4][e & 15], cs, -mc));
            asm volatile("" : "+v"(pe[e]));
            if (e >= 1) { tsum += pe[e - 1]; asm volatile("" : "+v"(tsum)); }
            if (e >= 2 && (e & 1) == 0) { pnew[(e - 2) >> 1] = pack2(pe[e - 2], pe[e - 1]); asm volatile("" : "+v"(pnew[(e - 2) >> 1])); }
            if (e >= 3 && (e & 1) == 1) { tsr = sum2(pnew[(e - 3) >> 1], tsr); asm volatile("" : "+v"(tsr)); }
        };
        // operand of slice i: 0..15 the V^T pieces of O^T += V(j-1)^T P(j-1)^T, 16..31 the K rows of
        // S(j+1) = K(j+1) Q^T, 32.. the next step's first V^T pieces
        auto fetch = [&](int i) -> bf16x8 {
            if (i < 16) return cat4(ldV(ldsV, i, 0), ldV(ldsV, i, 1));
            if (i < 32) return ldK(ldsK, i - 16);
            return cat4(ldV(ldsVn, i - 32, 0), ldV(ldsVn, i - 32, 1));
        };
        if (!SECOND) {
#pragma unroll
            for (int i = 0; i < RD - 1; ++i) ring[i] = fetch(i);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            if (i + RD - 1 < 32 || BRIDGE) ring[(i + RD - 1 + OFF) % RD] = fetch(i + RD - 1);
            if (i < 16)     // P operand outermost so that its registers die early
                oacc[i & 3] = mfma32(ring[(i + OFF) % RD], pbop(pbw, i >> 3, (i >> 2) & 1), oacc[i & 3]);
            else
                Snext[(i - 16) >> 3] = mfma32(ring[(i + OFF) % RD], qreg[i & 7], (i & 7) == 0 ? zero16 : Snext[(i - 16) >> 3]);
            valu(i);
            __builtin_amdgcn_sched_barrier(0);
        }
        tsum += pe[31];
        pnew[15] = pack2(pe[30], pe[31]);
        tsr = sum2(pnew[15], tsr);
        if (__builtin_amdgcn_ballot_w64(!(tsum <= P_LIMIT)) != 0) {
            float mx = Scur[0][0];
#pragma unroll
            for (int e = 1; e < 32; ++e) mx = fmaxf(mx, Scur[e >> 4][e & 15]);
            mx = pair_max(mx);
            const float mnew = fmaxf(m, mx);          // m is always finite
            const float alpha = __builtin_amdgcn_exp2f((m - mnew) * cs);
            lsum *= alpha;
            lsr *= alpha;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
            m = mnew;
            const float mc2 = mnew * cs;
            tsum = 0.f;
            tsr = 0.f;
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(Scur[q >> 3][(2 * q) & 15], cs, -mc2));
                const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(Scur[q >> 3][((2 * q) & 15) + 1], cs, -mc2));
                tsum += p0 + p1;
                pnew[q] = pack2(p0, p1);
                tsr = sum2(pnew[q], tsr);
            }
        }
        lsum += tsum;
        lsr += tsr;
    };

    // Zero-fill every V buffer that is multiplied against P = 0 before a copy has filled it: the last
    // buffer stands for V(-1) in the first step, and a key loop shorter than the buffer ring is still
    // padded to a whole turn of it, whose later V tiles are never copied.  LDS keeps what earlier
    // workgroups left there (bit patterns that may read as inf or NaN), and 0 * NaN would reach O.
#pragma unroll
    for (int b = 1; b < NB; ++b)
        if (b == NB - 1 || total <= b)
            for (int i = tid; i < TILE_BYTES / 16; i += 64 * NW)
                reinterpret_cast<i32x4*>(ldsVb[b])[i] = i32x4{0, 0, 0, 0};
    if constexpr (NB == 4) {
        issue(kbase_s, m0K[0], 0);
        issue(kbase_s, m0K[1], 1);
        issue(kbase_s, m0K[2], 2);
        issue(vbase_s, m0V[0], 0);
    } else {
        issue(kbase_s, m0K[0], 0);
        issue(kbase_s, m0K[1], 1);
    }
    wait_vm0();
    __syncthreads();
    qk_plain(ldsKb[0], sA);
    {   // exact row maximum of the first tile as the initial reference point
        if (needs_mask(0)) mask(0, sA);
        float mx = sA[0][0];
#pragma unroll
        for (int e = 1; e < 32; ++e) mx = fmaxf(mx, sA[e >> 4][e & 15]);
        mx = pair_max(mx);
        // A row that sees nothing in this tile (possible only without a prompt: a later response's
        // rows against the first response's keys) starts from a finite sentinel far below any score:
        // the first tile in which it does see a key then overflows the after-check and takes that
        // tile's exact maximum.  (Starting from 0 would let a row whose scores all lie below about
        // -126 / log2(e) underflow to a zero sum.)
        m = (mx == -INFINITY) ? M_NONE : mx;
    }
    if constexpr (NB == 4) {
        // Two steps per workgroup barrier: with four K and four V buffers the tiles of the next two
        // steps are copied while these two run.  At the barrier before steps j, j+1 (j even) the tiles
        // V(j-1), V(j), K(j+1), K(j+2) are resident and V(j+1), V(j+2), K(j+3), K(j+4) are issued into
        // the four buffers that the previous two steps read last.  The loop is padded to a multiple of
        // four steps (buffer indices are compile-time); padded steps are fully masked.
        const int total4 = (total + 3) & ~3;
        for (int j = 0; j < total4; j += 4) {
            wait_vm0();
            __syncthreads();
            issue(vbase_s, m0V[1], j + 1);
            issue(vbase_s, m0V[2], j + 2);
            issue(kbase_s, m0K[3], j + 3);
            issue(kbase_s, m0K[0], j + 4);
            step(j, std::integral_constant<int, 0>{}, std::false_type{}, std::true_type{}, sA, sB, pbA, pbB);
            step(j + 1, std::integral_constant<int, 1>{}, std::true_type{}, std::false_type{}, sB, sA, pbB, pbA);
            wait_vm0();
            __syncthreads();
            issue(vbase_s, m0V[3], j + 3);
            issue(vbase_s, m0V[0], j + 4);
            issue(kbase_s, m0K[1], j + 5);
            issue(kbase_s, m0K[2], j + 6);
            step(j + 2, std::integral_constant<int, 2>{}, std::false_type{}, std::true_type{}, sA, sB, pbA, pbB);
            step(j + 3, std::integral_constant<int, 3>{}, std::true_type{}, std::false_type{}, sB, sA, pbB, pbA);
        }
    } else {
        // One step per barrier.  At the barrier before step j the tiles V(j-1) and K(j+1) are resident
        // (issued a whole step earlier); V(j) and K(j+2) are issued into the buffers that step j-1 read
        // last (V(j-2), and K(j), from which S(j) has been formed).  Padded to an even count of steps.
        const int total2 = (total + 1) & ~1;
        for (int j = 0; j < total2; j += 2) {
            wait_vm0();
            __syncthreads();
            issue(vbase_s, m0V[0], j);
            issue(kbase_s, m0K[0], j + 2);
            step(j, std::integral_constant<int, 0>{}, std::false_type{}, std::false_type{}, sA, sB, pbA, pbB);
            wait_vm0();
            __syncthreads();
            issue(vbase_s, m0V[1], j + 1);
            issue(kbase_s, m0K[1], j + 3);
            step(j + 1, std::integral_constant<int, 1>{}, std::false_type{}, std::false_type{}, sB, sA, pbB, pbA);
        }
    }
    wait_vm0();
    __syncthreads();
    // lane indices re-derived behind an opaque barrier: the addresses of everything behind the loop are
    // loop-invariant, and hoisted above the main loop they would cost it registers (they were spilled)
    int lz = l;
    asm volatile("" : "+v"(lz));
    {   // P of the last (padded) step and its V tile
        const int c16z = (lz >> 4) & 1, j16z = lz & 15, hhz = lz >> 5;
        const char* ldsV = ldsVb[NB - 1];
        auto ldVz = [&](int i, int half) -> s16x4 {
            const int col4 = 32 * (i & 3) + 16 * c16z + 4 * (j16z & 3);
            const int row4 = 32 * (i >> 3) + 16 * ((i >> 2) & 1) + 4 * hhz + (j16z >> 2) + 8 * half;
            return lds_read_tr4(ldsV, row4, col4);
        };
        s16x4 rg[RD][2];
#pragma unroll
        for (int i = 0; i < RD - 1; ++i) { rg[i][0] = ldVz(i, 0); rg[i][1] = ldVz(i, 1); }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if (i + RD - 1 < 16) { rg[(i + RD - 1) % RD][0] = ldVz(i + RD - 1, 0); rg[(i + RD - 1) % RD][1] = ldVz(i + RD - 1, 1); }
            oacc[i & 3] = mfma32(cat4(rg[i % RD][0], rg[i % RD][1]), pbop(pbA, i >> 3, (i >> 2) & 1), oacc[i & 3]);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // O is normalised by the sum of the ROUNDED weights, the ones V was actually multiplied by:
    // a row dominated by one key then returns that key's V exactly, whatever the reference point.
    // LSE uses the unrounded sum.
    const float ltot = pair_sum(lsum);
    const float lrt = pair_sum(lsr);
    // The K buffers are free from here on (every wave has passed the last barrier and only the last V buffer
    // is still read).  A lane holds 16 pieces of 8 bytes of its row; written to memory directly, one
    // store instruction would touch 32 rows.  Each wave therefore stages its own 32 rows x 256 B in
    // its own 8 KB of LDS (swizzled like the operand tiles: two-way conflicts on the 8-byte writes,
    // which is their minimum, none on the 16-byte reads) and stores whole rows: 16 lanes per row,
    // four rows per instruction.  No workgroup barrier: a wave reads back only what it wrote.
    char* const stage = ldsKb[0] + 8192 * w;
    const float inv = 1.0f / lrt;
    auto store_rows = [&, c = lz & 31, hh = lz >> 5, l = lz](__bf16* dst, auto value) {
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                bf16x4 x;
#pragma unroll
                for (int e = 0; e < 4; ++e) x[e] = value(db, 4 * gq + e);
                *reinterpret_cast<bf16x4*>(stage + tile_off(c, 4 * db + gq) + 8 * hh) = x;
            }
        // all eight reads first, then the stores (one LDS round trip instead of eight); the rows of one lane lie
        // four rows apart, so one 64-bit address and a constant stride serve all of them
        bf16x8 x[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] = lds_read_row8(stage, 4 * i + (l >> 4), l & 15);
        __builtin_amdgcn_sched_barrier(0);
        __bf16* const p0 = dst + ((int64_t)(gd.tok_base + tw0 + (l >> 4)) * a.Hq + head) * 128 + 8 * (l & 15);
        const int64_t stride = (int64_t)4 * a.Hq * 128;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int tr = tw0 + 4 * i + (l >> 4);
            if (tr < Tg && !(a.resp_only && tr < Lp)) *reinterpret_cast<bf16x8*>(p0 + i * stride) = x[i];
        }
    };
    store_rows(ao, [&](int db, int r) { return (__bf16)(oacc[db][r] * inv); });
    if (a.o_lo)              // what the rounding of o dropped: lets the backward form D from an unrounded o
        store_rows(a.o_lo, [&](int db, int r) {
            const float x = oacc[db][r] * inv;
            return (__bf16)(x - (float)(__bf16)x);
        });
    if (valid && !(a.resp_only && t < Lp) && hh == 0)
        alse[(int64_t)head * T_total + gd.tok_base + t] = (m * cs + __log2f(ltot)) * LN2;
}

}  // namespace

hipError_t launch_fwd_bf16(const Problem& p, hipStream_t s) {
    FwdArgs a{};
    const int n_sets = p.n_sets > 1 ? p.n_sets : 1;
    for (int i = 0; i < n_sets; ++i) {
        const bool multi = p.n_sets > 1;
        a.q[i] = (const __bf16*)(multi ? p.qs[i] : p.q); a.k[i] = (const __bf16*)(multi ? p.ks[i] : p.k);
        a.v[i] = (const __bf16*)(multi ? p.vs[i] : p.v);
        a.o[i] = (__bf16*)(multi ? p.os[i] : p.o_out); a.lse[i] = multi ? p.lses[i] : p.lse_out;
    }
    a.tab = p.tab; a.n_groups = p.n_groups; a.sched = p.sched;
    a.Hq = p.Hq; a.Hkv = p.Hkv; a.c = p.scale * LOG2E; a.naive = p.naive; a.resp_only = p.resp_only;
    a.o_lo = n_sets == 1 ? (__bf16*)p.o_lo_out : nullptr;
    // Short key loops: the 128-row shape, two workgroups per CU (see fwd_kernel).  The naive baseline keeps
    // the 256-row shape whatever the packing (its loops are long by construction).
    const bool small = !p.naive && use_small_shape(p);
    const int bm = small ? 128 : 256;
    a.n_tiles = count_tiles(p, bm);
    a.blocks_per_set = grid_for_items(a.n_tiles, p.Hq, p.Hkv);
    if (a.blocks_per_set % 8 != 0) a.blocks_per_set += 8 - a.blocks_per_set % 8;
    if (p.naive) hipLaunchKernelGGL((fwd_kernel<8, true>), dim3(a.blocks_per_set * n_sets), dim3(512), 0, s, a);
    else if (small) hipLaunchKernelGGL((fwd_kernel<4, false>), dim3(a.blocks_per_set * n_sets), dim3(256), 0, s, a);
    else hipLaunchKernelGGL((fwd_kernel<8, false>), dim3(a.blocks_per_set * n_sets), dim3(512), 0, s, a);
    return hipGetLastError();
}

}  // namespace sp
