// Shared device-side definitions for the shared-prompt attention kernels (gfx950 only).
//
// Packed layout and mask follow Section 4.3 of the paper: a group is
// [prompt | resp_1 | ... | resp_G]; query t may attend key s iff s <= t and
// (s is a prompt token or s lies in t's own response).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));

// ---------------------------------------------------------------------------
// Segment table (int32 words, device memory, written by sp_upload_table):
//   [0] n_groups   [1] total_tokens   [2] table_words   [3] reserved
//   group g at 4 + 8*g : { tok_base, prompt_len, T_g, roff_idx, G, tiles256_before, tiles128_before, reserved }
//   roff_idx points at G+1 group-local offsets: roff[0] = prompt_len,
//   roff[i+1] = roff[i] + len(resp_i), roff[G] = T_g.
//   tilesB_before = sum over earlier groups of ceil(T_g / B): the kernels number their work
//   tiles (B rows or keys) group by group and find a tile's group by bisection on this word.
// ---------------------------------------------------------------------------
constexpr int TAB_HEADER = 4;
constexpr int TAB_GROUP_WORDS = 8;
constexpr int TAB_TILES256 = 5;        // word of the group entry: 256-row tiles before this group
constexpr int TAB_TILES128 = 6;        // 128-key tiles before this group
constexpr int TAB_CHUNK_WORDS = 960;   // words carried by one upload launch (kernarg limit 4 KB)

struct TabChunk { int32_t w[TAB_CHUNK_WORDS]; };
constexpr int PREP_WORDS = 896;        // largest table that travels beside the other arguments of the one-launch preparation
struct PrepChunk { int32_t w[PREP_WORDS]; };

struct GroupDesc {
    int tok_base;       // first packed token of the group
    int Lp;             // prompt length
    int Tg;             // tokens in the group
    int G;              // number of responses
    const int* roff;    // G+1 group-local response offsets
};

__device__ __forceinline__ GroupDesc load_group(const int* __restrict__ tab, int g) {
    const int* e = tab + TAB_HEADER + TAB_GROUP_WORDS * g;
    GroupDesc d;
    d.tok_base = e[0]; d.Lp = e[1]; d.Tg = e[2]; d.roff = tab + e[3]; d.G = e[4];
    return d;
}

// Start of the segment that owns group-local token t: 0 for a prompt token, the first
// token of its response otherwise.  Requires 0 <= t < Tg.  With this value the mask is
//   allowed(t, s) = (s <= t) && (s < Lp || s >= seg_start(t)).
__device__ __forceinline__ int seg_start(const GroupDesc& d, int t) {
    if (t < d.Lp) return 0;
    int lo = 0, hi = d.G;              // invariant: roff[lo] <= t, (hi == G or roff[hi] > t)
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (d.roff[mid] <= t) lo = mid; else hi = mid;
    }
    return d.roff[lo];
}

// One past the last token of the segment that owns t (prompt: Lp).
__device__ __forceinline__ int seg_end(const GroupDesc& d, int t) {
    if (t < d.Lp) return d.Lp;
    int lo = 0, hi = d.G;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (d.roff[mid] <= t) lo = mid; else hi = mid;
    }
    return d.roff[lo + 1];
}

// Segment bounds [st, en) of N group-local response tokens at once (every t[n] must satisfy
// Lp <= t[n] < Tg; for a prompt token the caller substitutes its own bounds).  One descending-step
// search over the response offsets per token, all N advanced in lock-step with unconditional
// loads, so the N dependent load chains overlap instead of following one another.  st is the last
// accepted offset; en is the last rejected one (the probes that fail come at ever smaller indices,
// the last of them is the accepted index + 1), so neither needs a load after the search.
template <int N>
__device__ __forceinline__ void seg_bounds(const GroupDesc& d, const int (&t)[N], int (&st)[N], int (&en)[N]) {
    int pos[N];
#pragma unroll
    for (int n = 0; n < N; ++n) { pos[n] = 0; st[n] = d.Lp; en[n] = d.Tg; }
    for (int step = d.G > 0 ? 1 << (31 - __clz(d.G)) : 0; step >= 1; step >>= 1) {
        int val[N];
#pragma unroll
        for (int n = 0; n < N; ++n) val[n] = d.roff[pos[n] + step < d.G ? pos[n] + step : 0];
#pragma unroll
        for (int n = 0; n < N; ++n) {
            const bool in = pos[n] + step < d.G;
            if (in && val[n] <= t[n]) { pos[n] += step; st[n] = val[n]; }
            else if (in) en[n] = val[n];
        }
    }
}

// Group that owns packed token tok (0 <= tok < total_tokens): bisection on tok_base.
__device__ __forceinline__ int find_group_of_token(const int* __restrict__ tab, int64_t tok) {
    int lo = 0, hi = tab[0];           // invariant: tok_base[lo] <= tok, (hi == n_groups or tok_base[hi] > tok)
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (tab[TAB_HEADER + TAB_GROUP_WORDS * mid] <= tok) lo = mid; else hi = mid;
    }
    return lo;
}

// Work-tile lookup: tiles of BT rows (256) or keys (128) are numbered group by group.  Returns
// the group and the tile's index inside it (0 .. ceil(T_g / BT) - 1), or g_out = -1 when the
// tile number lies past the last group.  Bisection on the group entries' running tile counts,
// so a batch of many small groups costs log2(n_groups) dependent scalar loads per workgroup.
template <int BT>
__device__ __forceinline__ void find_tile(const int* __restrict__ tab, int n_groups, int tile, int& g_out, int& idx_out) {
    static_assert(BT == 256 || BT == 128, "the table carries running tile counts for 256 and 128 only");
    constexpr int W = BT == 256 ? TAB_TILES256 : TAB_TILES128;
    int lo = 0, hi = n_groups;         // passed in (a kernel argument): one load less at the head of the chain
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (tab[TAB_HEADER + TAB_GROUP_WORDS * mid + W] <= tile) lo = mid; else hi = mid;
    }
    const int* e = tab + TAB_HEADER + TAB_GROUP_WORDS * lo;
    const int idx = tile - e[W];
    const int nt = (e[2] + BT - 1) / BT;
    g_out = idx < nt ? lo : -1;
    idx_out = idx;
}

// Schedule: what the MFMA kernels' prologues would otherwise look up in the table through chains of
// dependent loads, written once per call by a small kernel (sp_f32.hip: schedule_kernel).
//   TileDesc  per work tile (one array for tiles of 256, one for tiles of 128 rows or keys): its group
//             and index inside the group, and the group's first token, prompt length and token count
//   key_lo[tok]  first key of its own segment that token tok may attend besides the prompt
//                (group-local; 0 for a prompt token): the mask is s <= t && (s < Lp || s >= key_lo[t])
//   row_hi[tok]  one past the last row that sees token tok as a key (group-local): the group's end for
//                a prompt token, the end of its response otherwise
struct TileDesc { int g, ti, tok_base, Lp, Tg, pad0, pad1, pad2; };
struct Schedule { const TileDesc* tiles256; const TileDesc* tiles128; const int* key_lo; const int* row_hi; };

// Map a flat block index to (tile, q head) so that the blocks an XCD receives
// (blocks are dealt round-robin over the 8 XCDs, each with a private L2) share one
// kv head, and q heads of the same tile sit next to each other.
// Returns false when the block has no work.
__device__ __forceinline__ bool decode_item(int bid, int n_tiles, int Hq, int Hkv,
                                            int& tile, int& head) {
    const int rep = Hq / Hkv;
    const int per_kv = n_tiles * rep;          // items of one kv head
    if (Hkv % 8 == 0) {
        const int x = bid & 7, j = bid >> 3;
        const int kv_per_x = Hkv >> 3;
        const int hr = j % rep;
        const int rest = j / rep;
        const int kvl = rest % kv_per_x;
        tile = rest / kv_per_x;
        head = (x + 8 * kvl) * rep + hr;
        return tile < n_tiles;
    }
    if (8 % Hkv == 0) {
        const int nx = 8 / Hkv;                // XCDs that share one kv head
        const int x = bid & 7, j = bid >> 3;
        const int kvh = x / nx, sub = x % nx;
        const int it = j * nx + sub;
        if (it >= per_kv) return false;
        tile = it / rep;
        head = kvh * rep + it % rep;
        return true;
    }
    tile = bid / Hq;
    head = bid % Hq;
    return tile < n_tiles;
}

__host__ __device__ inline int grid_for_items(int n_tiles, int Hq, int Hkv) {
    const int rep = Hq / Hkv;
    if (Hkv % 8 == 0) return 8 * (n_tiles * rep * (Hkv / 8));
    if (8 % Hkv == 0) { const int nx = 8 / Hkv; return 8 * ((n_tiles * rep + nx - 1) / nx); }
    return n_tiles * Hq;
}

// ---------------------------------------------------------------------------
// LDS tiles: rows of 128 bf16 (256 B = 16 granules of 16 B).  Granule g of row r is
// stored at granule slot g ^ swz(r).  swz permutes 0..15 over 16 consecutive rows
// (conflict-free b128 reads of one granule column by 16 rows) and its two high bits
// differ over 4 consecutive rows (conflict-free transposed b64 reads of a 4-row x
// 4-granule block).
// ---------------------------------------------------------------------------
__device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

__device__ __forceinline__ int tile_off(int row, int granule) {   // byte offset
    return row * 256 + ((granule ^ swz(row)) << 4);
}

typedef __attribute__((address_space(3))) char lds_char;

__device__ __forceinline__ bf16x8 lds_read_row8(const char* tile, int row, int granule) {
    return *reinterpret_cast<const bf16x8*>(tile + tile_off(row, granule));
}

// Transposed read feeding an MFMA operand whose in-lane (contraction) index runs over
// tile ROWS: the lane receives rows row4 .. row4+3 at column col (one bf16 each).
// Lanes of a 16-lane group must pass: row = row4 + (j >> 2), col4 = colbase + 4*(j & 3)
// with j = lane & 15; lane j then receives column colbase + j.
__device__ __forceinline__ s16x4 lds_read_tr4(const char* tile, int row, int col4) {
    const char* p = tile + tile_off(row, col4 >> 3) + ((col4 & 4) << 1);
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) s16x4*)(p));
}

__device__ __forceinline__ bf16x8 cat4(s16x4 a, s16x4 b) {
    s16x8 r = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
}

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Round 8 floats to bf16 (round-to-nearest-even, hardware v_cvt_pk_bf16_f32).
__device__ __forceinline__ bf16x8 pack8(float a0, float a1, float a2, float a3,
                                        float a4, float a5, float a6, float a7) {
    bf16x8 r;
    r[0] = (__bf16)a0; r[1] = (__bf16)a1; r[2] = (__bf16)a2; r[3] = (__bf16)a3;
    r[4] = (__bf16)a4; r[5] = (__bf16)a5; r[6] = (__bf16)a6; r[7] = (__bf16)a7;
    return r;
}

__device__ __forceinline__ float xor32(float x) { return __shfl_xor(x, 32, 64); }

// max / sum of x over the lane pair (l, l ^ 32) with one v_permlane32_swap: after the swap
// one result holds the low-half value and the other the high-half value in every lane.
__device__ __forceinline__ float pair_max(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pair_sum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Asynchronous global -> LDS copy of 16 bytes per lane (global_load_lds_dwordx4): lane i of
// the wave writes LDS bytes [lds_base + 16*i, +16).  lds_base must be wave-uniform.
// Written as inline assembly so that the compiler does not place a conservative
// "wait for all global loads" in front of every later LDS read; the kernels order the
// copy against its readers themselves with wait_vm0() followed by a workgroup barrier.
// M0 (the LDS base of the copy) is overwritten.  It cannot be named as a clobber: the compiler
// treats M0 as a reserved register (it rejects the clobber as undefined behaviour) and writes it
// itself immediately before each of its own uses, never keeping a value in it across statements;
// gfx9 LDS instructions do not read M0 and nothing else in these kernels uses it.
__device__ __forceinline__ void async_copy16(const void* gptr, char* lds_base) {
    const unsigned lds_addr = __builtin_amdgcn_readfirstlane(
        (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)lds_base);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :: "v"(gptr), "s"(lds_addr) : "memory");
}
// Same copy with the global address split into a wave-uniform 64-bit base (scalar registers)
// and a 32-bit per-lane byte offset, and the LDS destination given as a byte address: a kernel
// keeps the lane part constant and advances only the scalar base from tile to tile.
__device__ __forceinline__ void async_copy16_sm(uint64_t sbase, unsigned voff, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(sbase), "s"(lds_addr) : "memory");
}
// 4-byte variant: lane i writes LDS bytes [lds_base + 4*i, +4).
__device__ __forceinline__ void async_copy4(const void* gptr, char* lds_base) {
    const unsigned lds_addr = __builtin_amdgcn_readfirstlane(
        (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)lds_base);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off"
                 :: "v"(gptr), "s"(lds_addr) : "memory");
}
// wait until every global load (including global -> LDS copies) of this wave has landed
__device__ __forceinline__ void wait_vm0() { __builtin_amdgcn_s_waitcnt(0x0F70); }

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

}  // namespace sp
