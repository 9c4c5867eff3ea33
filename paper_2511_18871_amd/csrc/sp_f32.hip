// float32 plain-ALU debug path of shared-prompt attention, the segment-table upload
// and the backward preprocess D = rowsum(dO * O).
//
// The debug kernels give one wavefront a single (row, head) or (key, kv head) and walk
// the allowed keys / rows of the Section 4.3 mask in chunks of 64, one per lane.  No
// MFMA, no LDS: they exist to cross-check the MFMA path and to serve float32 callers.
#include "sp_common.hpp"
#include "sp_launch.hpp"
#include <type_traits>

namespace sp {
namespace {

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
    return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

__global__ void upload_table_kernel(TabChunk chunk, int* __restrict__ dst, int offset, int count) {
    for (int i = threadIdx.x; i < count; i += blockDim.x) dst[offset + i] = chunk.w[i];
}

// One thread per packed token writes its segment bounds, one per work tile its descriptor (see Schedule).
__device__ __forceinline__ void schedule_body(const int* __restrict__ tab, int n_groups, int64_t T_total, int n256,
                                              int n128, TileDesc* __restrict__ tiles256, TileDesc* __restrict__ tiles128,
                                              int* __restrict__ key_lo, int* __restrict__ row_hi) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < T_total) {
        const GroupDesc gd = load_group(tab, find_group_of_token(tab, i));
        const int t = (int)(i - gd.tok_base);
        int lo = 0, hi = gd.Tg;
        if (t >= gd.Lp) {
            const int tq[1] = {t};
            int sq[1], eq[1];
            seg_bounds<1>(gd, tq, sq, eq);
            lo = sq[0]; hi = eq[0];
        }
        key_lo[i] = lo;
        row_hi[i] = hi;
    }
    auto describe = [&](auto bt_tag, int n, TileDesc* out) {
        constexpr int BT = decltype(bt_tag)::value;
        if (i >= n) return;
        int g, ti;
        find_tile<BT>(tab, n_groups, (int)i, g, ti);
        if (g < 0) g = n_groups - 1;                   // cannot happen: n is the exact tile count
        const GroupDesc gd = load_group(tab, g);
        out[i] = TileDesc{g, ti, gd.tok_base, gd.Lp, gd.Tg, 0, 0, 0};
    };
    describe(std::integral_constant<int, 256>{}, n256, tiles256);
    describe(std::integral_constant<int, 128>{}, n128, tiles128);
}

__global__ __launch_bounds__(256) void schedule_kernel(const int* __restrict__ tab, int n_groups, int64_t T_total,
                                                       int n256, int n128, TileDesc* __restrict__ tiles256,
                                                       TileDesc* __restrict__ tiles128, int* __restrict__ key_lo,
                                                       int* __restrict__ row_hi) {
    schedule_body(tab, n_groups, T_total, n256, n128, tiles256, tiles128, key_lo, row_hi);
}

// Tag block maintenance, one wave.  See sp_launch.hpp for the modes.  A reserve written for all rows
// (word 10 = 0) also serves a backward over response rows only (want word 10 = 1), not the reverse.
__device__ __forceinline__ void reserve_tag_body(uint32_t* __restrict__ blk, const ReserveTag& want, int mode) {
    const int i = threadIdx.x;                  // one whole wave: lanes 0..63
    if (mode == TAG_CLEAR) { blk[i] = 0u; return; }
    if (mode == TAG_WRITE) { blk[i] = i < TAG_WORDS ? want.w[i] : 0u; return; }
    const uint32_t have = blk[i];
    bool same = i >= TAG_WORDS || have == want.w[i];
    if (i == 10) same = have == want.w[10] || have == 0u;
    const bool ok = __builtin_amdgcn_ballot_w64(!same) == 0;
    if (i < TAG_WORDS && !ok) blk[i] = 0u;
    if (i == TAG_FLAG_WORD) blk[i] = ok ? 1u : 0u;
}

__global__ __launch_bounds__(64) void reserve_tag_kernel(uint32_t* __restrict__ blk, ReserveTag want, int mode) {
    reserve_tag_body(blk, want, mode);
}

// Everything a call does ahead of its attention kernels, in one launch, for segment tables that fit one
// kernel-argument block: block 0 stores the table into the workspace and (first wave) maintains the tag
// block; every block works out its part of the schedule from a copy of the table in its own LDS, since the
// copy in memory is only complete when the kernel has ended.  Small problems, whose attention kernels run
// for tens of microseconds, otherwise spend a fifth of a call in three tiny launches and the gaps between them.
__global__ __launch_bounds__(256) void prepare_kernel(PrepChunk chunk, int n_words, int* __restrict__ dev_tab,
                                                      uint32_t* __restrict__ tag_blk, ReserveTag want, int tag_mode,
                                                      int with_schedule, int n_groups, int64_t T_total, int n256,
                                                      int n128, TileDesc* __restrict__ tiles256,
                                                      TileDesc* __restrict__ tiles128, int* __restrict__ key_lo,
                                                      int* __restrict__ row_hi) {
    __shared__ int tab_s[PREP_WORDS];
    for (int i = threadIdx.x; i < n_words; i += 256) {
        const int x = chunk.w[i];
        tab_s[i] = x;
        if (blockIdx.x == 0) dev_tab[i] = x;
    }
    if (blockIdx.x == 0 && threadIdx.x < 64 && tag_mode != TAG_KEEP) reserve_tag_body(tag_blk, want, tag_mode);
    __syncthreads();
    if (with_schedule) schedule_body(tab_s, n_groups, T_total, n256, n128, tiles256, tiles128, key_lo, row_hi);
}

template <typename T>
__global__ __launch_bounds__(256) void rowsum_kernel(const T* __restrict__ d_o, const T* __restrict__ o,
                                                     const float* __restrict__ lse, float* __restrict__ D,
                                                     int64_t T_total, int Hq, int dh,
                                                     const int* __restrict__ tab, int resp_only,
                                                     const T* __restrict__ o_lo) {
    const int64_t gw = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int l = threadIdx.x & 63;
    if (gw >= T_total * Hq) return;
    const int64_t tok = gw / Hq;
    const int h = (int)(gw % Hq);
    if (resp_only) {
        // prompt rows take no part: their o / lse may hold anything, so they are not read, and the
        // planes get finite placeholders (rows of a partly used tile are masked, not skipped)
        const GroupDesc gd = load_group(tab, find_group_of_token(tab, (int)tok));
        if ((int)tok - gd.tok_base < gd.Lp) {
            if (l == 0) {
                D[(int64_t)h * T_total + tok] = 0.f;
                D[(int64_t)Hq * T_total + (int64_t)h * T_total + tok] = 0.f;
            }
            return;
        }
    }
    const T* a = d_o + gw * dh;
    const T* b = o + gw * dh;
    float acc = 0.f;
    if (o_lo) {          // o was stored with its rounding residual: D from the unrounded value
        const T* c = o_lo + gw * dh;
        for (int i = l; i < dh; i += 64) acc += (float)a[i] * ((float)b[i] + (float)c[i]);
    } else {
        for (int i = l; i < dh; i += 64) acc += (float)a[i] * (float)b[i];
    }
    acc = wave_sum(acc);
    if (l == 0) {
        D[(int64_t)h * T_total + tok] = acc;
        // second plane: the row's logsumexp in base-2 units, as the MFMA backward consumes it
        D[(int64_t)Hq * T_total + (int64_t)h * T_total + tok] = lse[(int64_t)h * T_total + tok] * LOG2E;
    }
}

// The same rowsum for bf16 rows of 128 elements, laid out for bandwidth.  A block owns RS_TOK
// consecutive tokens x all q heads, which is one contiguous stretch of d_o and of o; 16 lanes read
// a (token, head) row as 16-byte pieces and add up over the lanes.  The sums pass through LDS so
// that each head's RS_TOK tokens leave as one contiguous store into the [Hq, T] planes.  In
// response-rows mode the prompt rows are still read (the buffers are whole) but their values are
// discarded by a select, never used in arithmetic that reaches the output.
constexpr int RS_TOK = 16;      // rowsum_fast_path() in sp_launch.hpp assumes this value
template <bool HAS_LO>
__global__ __launch_bounds__(256) void rowsum_bf16_kernel(const __bf16* __restrict__ d_o, const __bf16* __restrict__ o,
                                                          const float* __restrict__ lse, float* __restrict__ D,
                                                          int64_t T_total, int Hq, const int* __restrict__ tab,
                                                          int resp_only, const __bf16* __restrict__ o_lo,
                                                          const uint32_t* __restrict__ lo_flag) {
    extern __shared__ float rs_sum[];                  // [Hq][RS_TOK]
    __shared__ int rs_skip[RS_TOK];
    // the residual is the workspace's reserve: usable only if the tag check of this call said so
    const bool use_lo = HAS_LO && (lo_flag == nullptr || __builtin_amdgcn_readfirstlane((int)*lo_flag) != 0);
    const int64_t tok0 = (int64_t)blockIdx.x * RS_TOK;
    const int ntok = (int)(T_total - tok0 < RS_TOK ? T_total - tok0 : RS_TOK);
    const int tid = threadIdx.x, sub = tid & 15, grp = tid >> 4;
    if (tid < RS_TOK) {
        int sk = 0;
        if (resp_only && tid < ntok) {
            const GroupDesc gd = load_group(tab, find_group_of_token(tab, tok0 + tid));
            sk = (int)(tok0 + tid - gd.tok_base) < gd.Lp;
        }
        rs_skip[tid] = sk;
    }
    __syncthreads();
    const int nrows = ntok * Hq;
    const int64_t base = tok0 * Hq * 128 + 8 * sub;
    auto row_dot = [&](int r) -> float {
        const int64_t off = base + (int64_t)r * 128;
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(d_o + off);
        const bf16x8 b = *reinterpret_cast<const bf16x8*>(o + off);
        float acc = 0.f;
        if (HAS_LO && use_lo) {        // o was stored with its rounding residual: D from the unrounded value
            const bf16x8 c = *reinterpret_cast<const bf16x8*>(o_lo + off);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc = __builtin_fmaf((float)a[e], (float)b[e] + (float)c[e], acc);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) acc = __builtin_fmaf((float)a[e], (float)b[e], acc);
        }
        return acc;
    };
    auto put = [&](int r, float acc) {
#pragma unroll
        for (int sh = 8; sh >= 1; sh >>= 1) acc += __shfl_xor(acc, sh, 16);
        const int tl = r / Hq, h = r - tl * Hq;
        if (sub == 0) rs_sum[h * RS_TOK + tl] = rs_skip[tl] ? 0.f : acc;
    };
    for (int r = grp; r < nrows; r += 32) {            // two rows per trip: four to six loads in flight per lane
        const bool two = r + 16 < nrows;
        const float x0 = row_dot(r), x1 = row_dot(two ? r + 16 : r);
        put(r, x0);
        if (two) put(r + 16, x1);
    }
    __syncthreads();
    for (int i = tid; i < Hq * RS_TOK; i += 256) {
        const int h = i / RS_TOK, tl = i % RS_TOK;
        if (tl < ntok) {
            const int64_t idx = (int64_t)h * T_total + tok0 + tl;
            D[idx] = rs_sum[i];
            // second plane: the row's logsumexp in base-2 units, as the MFMA backward consumes it
            const float l2 = lse[idx] * LOG2E;
            D[(int64_t)Hq * T_total + idx] = rs_skip[tl] ? 0.f : l2;
        }
    }
}

template <int DH>
__device__ __forceinline__ float dot_row(const float* __restrict__ x, const float* __restrict__ y) {
    float acc = 0.f;
#pragma unroll 8
    for (int i = 0; i < DH; ++i) acc = __builtin_fmaf(x[i], y[i], acc);
    return acc;
}

template <int DH>
__global__ __launch_bounds__(256) void fwd_f32_kernel(const float* __restrict__ q, const float* __restrict__ k,
                                                      const float* __restrict__ v, float* __restrict__ o,
                                                      float* __restrict__ lse, const int* __restrict__ tab,
                                                      int Hq, int Hkv, float scale, int resp_only) {
    constexpr int PER = DH / 64;
    const int64_t T_total = tab[1];
    const int64_t gw = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int l = threadIdx.x & 63;
    if (gw >= T_total * Hq) return;
    const int tok = (int)(gw / Hq), h = (int)(gw % Hq);
    const GroupDesc gd = load_group(tab, find_group_of_token(tab, tok));
    const int t = tok - gd.tok_base;
    if (resp_only && t < gd.Lp) return;
    const int st = seg_start(gd, t);
    const int kvh = h / (Hq / Hkv);
    const float* qrow = q + ((int64_t)tok * Hq + h) * DH;
    const float* kb = k + ((int64_t)gd.tok_base * Hkv + kvh) * DH;
    const float* vb = v + ((int64_t)gd.tok_base * Hkv + kvh) * DH;
    const int64_t kvs = (int64_t)Hkv * DH;

    float m = -INFINITY, lsum = 0.f, acc[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) acc[e] = 0.f;
    for (int s0 = 0; s0 <= t; s0 += 64) {
        if (s0 >= gd.Lp && s0 + 64 <= st) continue;        // wholly inside other responses
        const int s = s0 + l;
        const bool ok = s <= t && (s < gd.Lp || s >= st);
        const float sc = ok ? scale * dot_row<DH>(qrow, kb + (int64_t)s * kvs) : -INFINITY;
        const float mnew = fmaxf(m, wave_max(sc));
        if (mnew == -INFINITY) continue;
        const float alpha = expf(m - mnew);
        const float p = ok ? expf(sc - mnew) : 0.f;
        lsum = lsum * alpha + wave_sum(p);
        m = mnew;
        const int nk = min(64, t + 1 - s0);
#pragma unroll
        for (int e = 0; e < PER; ++e) acc[e] *= alpha;
        for (int jj = 0; jj < nk; ++jj) {
            const float pj = __shfl(p, jj, 64);
            const float* vr = vb + (int64_t)(s0 + jj) * kvs;
#pragma unroll
            for (int e = 0; e < PER; ++e) acc[e] = __builtin_fmaf(pj, vr[l + 64 * e], acc[e]);
        }
    }
    float* orow = o + ((int64_t)tok * Hq + h) * DH;
#pragma unroll
    for (int e = 0; e < PER; ++e) orow[l + 64 * e] = acc[e] / lsum;
    if (l == 0) lse[(int64_t)h * T_total + tok] = m + logf(lsum);
}

// dQ[t,h] = scale * sum_s dS[t,s] K[s],  dS = P * (dP - D)
template <int DH>
__global__ __launch_bounds__(256) void bwd_dq_f32_kernel(const float* __restrict__ q, const float* __restrict__ k,
                                                         const float* __restrict__ v, const float* __restrict__ d_o,
                                                         const float* __restrict__ lse, const float* __restrict__ D,
                                                         float* __restrict__ dq, const int* __restrict__ tab,
                                                         int Hq, int Hkv, float scale, int resp_only) {
    constexpr int PER = DH / 64;
    const int64_t T_total = tab[1];
    const int64_t gw = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int l = threadIdx.x & 63;
    if (gw >= T_total * Hq) return;
    const int tok = (int)(gw / Hq), h = (int)(gw % Hq);
    const GroupDesc gd = load_group(tab, find_group_of_token(tab, tok));
    const int t = tok - gd.tok_base;
    if (resp_only && t < gd.Lp) return;
    const int st = seg_start(gd, t);
    const int kvh = h / (Hq / Hkv);
    const float* qrow = q + ((int64_t)tok * Hq + h) * DH;
    const float* gorow = d_o + ((int64_t)tok * Hq + h) * DH;
    const float* kb = k + ((int64_t)gd.tok_base * Hkv + kvh) * DH;
    const float* vb = v + ((int64_t)gd.tok_base * Hkv + kvh) * DH;
    const int64_t kvs = (int64_t)Hkv * DH;
    const float L = lse[(int64_t)h * T_total + tok];
    const float Dt = D[(int64_t)h * T_total + tok];

    float acc[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) acc[e] = 0.f;
    for (int s0 = 0; s0 <= t; s0 += 64) {
        if (s0 >= gd.Lp && s0 + 64 <= st) continue;
        const int s = s0 + l;
        const bool ok = s <= t && (s < gd.Lp || s >= st);
        float ds = 0.f;
        if (ok) {
            const float p = expf(scale * dot_row<DH>(qrow, kb + (int64_t)s * kvs) - L);
            ds = p * (dot_row<DH>(gorow, vb + (int64_t)s * kvs) - Dt);
        }
        const int nk = min(64, t + 1 - s0);
        for (int jj = 0; jj < nk; ++jj) {
            const float dj = __shfl(ds, jj, 64);
            const float* kr = kb + (int64_t)(s0 + jj) * kvs;
#pragma unroll
            for (int e = 0; e < PER; ++e) acc[e] = __builtin_fmaf(dj, kr[l + 64 * e], acc[e]);
        }
    }
    float* out = dq + ((int64_t)tok * Hq + h) * DH;
#pragma unroll
    for (int e = 0; e < PER; ++e) out[l + 64 * e] = scale * acc[e];
}

// dK[s,g] = scale * sum_{h in g} sum_t dS[t,s] Q[t,h];  dV[s,g] = sum_{h in g} sum_t P[t,s] dO[t,h].
// The rows that see key s are contiguous: [s, Tg) for a prompt key (later prompt rows and
// every row of every response), [s, end of its response) otherwise.
template <int DH>
__global__ __launch_bounds__(256) void bwd_dkdv_f32_kernel(const float* __restrict__ q, const float* __restrict__ k,
                                                           const float* __restrict__ v, const float* __restrict__ d_o,
                                                           const float* __restrict__ lse, const float* __restrict__ D,
                                                           float* __restrict__ dk, float* __restrict__ dv,
                                                           const int* __restrict__ tab, int Hq, int Hkv, float scale,
                                                           int resp_only, int accumulate) {
    constexpr int PER = DH / 64;
    const int64_t T_total = tab[1];
    const int64_t gw = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int l = threadIdx.x & 63;
    if (gw >= T_total * Hkv) return;
    const int tok = (int)(gw / Hkv), kvh = (int)(gw % Hkv);
    const GroupDesc gd = load_group(tab, find_group_of_token(tab, tok));
    const int s = tok - gd.tok_base;
    const int row_end = s < gd.Lp ? gd.Tg : seg_end(gd, s);
    const int rep = Hq / Hkv;
    const float* krow = k + ((int64_t)tok * Hkv + kvh) * DH;
    const float* vrow = v + ((int64_t)tok * Hkv + kvh) * DH;

    float ak[PER], av[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) { ak[e] = 0.f; av[e] = 0.f; }
    for (int hr = 0; hr < rep; ++hr) {
        const int h = kvh * rep + hr;
        for (int r0 = resp_only ? max(s, gd.Lp) : s; r0 < row_end; r0 += 64) {
            const int t = r0 + l;
            float p = 0.f, ds = 0.f;
            if (t < row_end) {
                const int64_t row = ((int64_t)(gd.tok_base + t) * Hq + h) * DH;
                const int64_t sidx = (int64_t)h * T_total + gd.tok_base + t;
                p = expf(scale * dot_row<DH>(q + row, krow) - lse[sidx]);
                ds = p * (dot_row<DH>(d_o + row, vrow) - D[sidx]);
            }
            const int nr = min(64, row_end - r0);
            for (int jj = 0; jj < nr; ++jj) {
                const float pj = __shfl(p, jj, 64), dj = __shfl(ds, jj, 64);
                const int64_t row = ((int64_t)(gd.tok_base + r0 + jj) * Hq + h) * DH;
#pragma unroll
                for (int e = 0; e < PER; ++e) {
                    av[e] = __builtin_fmaf(pj, d_o[row + l + 64 * e], av[e]);
                    ak[e] = __builtin_fmaf(dj, q[row + l + 64 * e], ak[e]);
                }
            }
        }
    }
    float* okr = dk + ((int64_t)tok * Hkv + kvh) * DH;
    float* ovr = dv + ((int64_t)tok * Hkv + kvh) * DH;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        okr[l + 64 * e] = scale * ak[e] + (accumulate ? okr[l + 64 * e] : 0.f);
        ovr[l + 64 * e] = av[e] + (accumulate ? ovr[l + 64 * e] : 0.f);
    }
}

inline int blocks_for_waves(int64_t waves) { return (int)((waves + 3) / 4); }

}  // namespace

// Tag block, segment table and (bf16) schedule of a call: one launch when the table fits a kernel-argument
// block, else the tag kernel, the table in pieces and the schedule kernel.
hipError_t launch_prepare(const int32_t* host_words, int n_words, int* dev_tab, uint32_t* tag_block, const ReserveTag& tag,
                          int tag_mode, bool with_schedule, int n_groups, int64_t total_tokens, int n256, int n128,
                          const Schedule& sched, hipStream_t s) {
    TileDesc* const t256 = (TileDesc*)sched.tiles256;
    TileDesc* const t128 = (TileDesc*)sched.tiles128;
    int* const key_lo = (int*)sched.key_lo;
    int* const row_hi = (int*)sched.row_hi;
    int64_t n = total_tokens;
    if (n128 > n) n = n128;                            // n128 >= n256
    const unsigned sched_blocks = (unsigned)((n + 255) / 256);
    if (n_words <= PREP_WORDS) {
        PrepChunk c;
        for (int i = 0; i < n_words; ++i) c.w[i] = host_words[i];
        for (int i = n_words; i < PREP_WORDS; ++i) c.w[i] = 0;
        hipLaunchKernelGGL(prepare_kernel, dim3(with_schedule ? sched_blocks : 1u), dim3(256), 0, s, c, n_words, dev_tab,
                           tag_block, tag, tag_mode, with_schedule ? 1 : 0, n_groups, total_tokens, n256, n128, t256, t128,
                           key_lo, row_hi);
        return hipGetLastError();
    }
    if (tag_mode != TAG_KEEP) {
        hipLaunchKernelGGL(reserve_tag_kernel, dim3(1), dim3(64), 0, s, tag_block, tag, tag_mode);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    for (int off = 0; off < n_words; off += TAB_CHUNK_WORDS) {
        TabChunk c;
        const int nw = n_words - off < TAB_CHUNK_WORDS ? n_words - off : TAB_CHUNK_WORDS;
        for (int i = 0; i < nw; ++i) c.w[i] = host_words[off + i];
        for (int i = nw; i < TAB_CHUNK_WORDS; ++i) c.w[i] = 0;
        hipLaunchKernelGGL(upload_table_kernel, dim3(1), dim3(256), 0, s, c, dev_tab, off, nw);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (with_schedule)
        hipLaunchKernelGGL(schedule_kernel, dim3(sched_blocks), dim3(256), 0, s, (const int*)dev_tab, n_groups, total_tokens,
                           n256, n128, t256, t128, key_lo, row_hi);
    return hipGetLastError();
}

hipError_t launch_rowsum(const Problem& p, bool f32, hipStream_t s) {
    const int grid = blocks_for_waves(p.total_tokens * p.Hq);
    if (f32)
        hipLaunchKernelGGL(rowsum_kernel<float>, dim3(grid), dim3(256), 0, s, (const float*)p.d_o,
                           (const float*)p.o, p.lse, p.Dbuf, p.total_tokens, p.Hq, p.head_dim, p.tab, p.resp_only, (const float*)nullptr);
    else if (rowsum_fast_path(p)) {
        const dim3 g((unsigned)((p.total_tokens + RS_TOK - 1) / RS_TOK));
        const size_t lds = (size_t)p.Hq * RS_TOK * sizeof(float);
        if (p.o_lo)
            hipLaunchKernelGGL(rowsum_bf16_kernel<true>, g, dim3(256), lds, s, (const __bf16*)p.d_o, (const __bf16*)p.o,
                               p.lse, p.Dbuf, p.total_tokens, p.Hq, p.tab, p.resp_only, (const __bf16*)p.o_lo, p.o_lo_flag);
        else
            hipLaunchKernelGGL(rowsum_bf16_kernel<false>, g, dim3(256), lds, s, (const __bf16*)p.d_o, (const __bf16*)p.o,
                               p.lse, p.Dbuf, p.total_tokens, p.Hq, p.tab, p.resp_only, (const __bf16*)nullptr,
                               (const uint32_t*)nullptr);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        // exact D for the rows that see only a few keys (sp_edge.hip)
        e = launch_short_rows(p, false, s);
        if (e != hipSuccess) return e;
    }
    else
        hipLaunchKernelGGL(rowsum_kernel<__bf16>, dim3(grid), dim3(256), 0, s, (const __bf16*)p.d_o,
                           (const __bf16*)p.o, p.lse, p.Dbuf, p.total_tokens, p.Hq, p.head_dim, p.tab, p.resp_only,
                           (const __bf16*)(p.o_lo_flag ? nullptr : p.o_lo));      // this fallback does not consult the reserve
    return hipGetLastError();
}

hipError_t launch_fwd_f32(const Problem& p, hipStream_t s) {
    const int grid = blocks_for_waves(p.total_tokens * p.Hq);
    if (p.head_dim == 64)
        hipLaunchKernelGGL(fwd_f32_kernel<64>, dim3(grid), dim3(256), 0, s, (const float*)p.q, (const float*)p.k,
                           (const float*)p.v, (float*)p.o_out, p.lse_out, p.tab, p.Hq, p.Hkv, p.scale, p.resp_only);
    else
        hipLaunchKernelGGL(fwd_f32_kernel<128>, dim3(grid), dim3(256), 0, s, (const float*)p.q, (const float*)p.k,
                           (const float*)p.v, (float*)p.o_out, p.lse_out, p.tab, p.Hq, p.Hkv, p.scale, p.resp_only);
    return hipGetLastError();
}

hipError_t launch_bwd_f32(const Problem& p, hipStream_t s) {
    if (p.stages & STAGE_ROWSUM) {
        hipError_t e = launch_rowsum(p, true, s);
        if (e != hipSuccess) return e;
    }
    const int gq = blocks_for_waves(p.total_tokens * p.Hq);
    const int gk = blocks_for_waves(p.total_tokens * p.Hkv);
#define SP_F32_BWD(DH)                                                                                      \
    if (p.stages & STAGE_DQ)                                                                               \
    hipLaunchKernelGGL(bwd_dq_f32_kernel<DH>, dim3(gq), dim3(256), 0, s, (const float*)p.q, (const float*)p.k, \
                       (const float*)p.v, (const float*)p.d_o, p.lse, p.Dbuf, (float*)p.dq, p.tab, p.Hq,   \
                       p.Hkv, p.scale, p.resp_only);                                                       \
    if (p.stages & STAGE_DKDV)                                                                             \
    hipLaunchKernelGGL(bwd_dkdv_f32_kernel<DH>, dim3(gk), dim3(256), 0, s, (const float*)p.q,              \
                       (const float*)p.k, (const float*)p.v, (const float*)p.d_o, p.lse, p.Dbuf,           \
                       (float*)p.dk, (float*)p.dv, p.tab, p.Hq, p.Hkv, p.scale, p.resp_only, p.accumulate);
    if (p.head_dim == 64) { SP_F32_BWD(64) } else { SP_F32_BWD(128) }
#undef SP_F32_BWD
    return hipGetLastError();
}

}  // namespace sp
