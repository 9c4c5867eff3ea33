// C-ABI entry points of the shared-prompt attention library: argument validation,
// segment-table construction and kernel dispatch.  See include/sp_attn.h for the contract.
#include "../../include/sp_attn.h"
#include "sp_common.hpp"
#include "sp_launch.hpp"

#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <vector>

// Device memory of the entry point that takes no workspace (sp_attn_bwd_batched_static): segment
// table, D and scaled-LSE planes and, on small problems, the per-q-head dK/dV partial sums.  Every
// GPU the library runs on holds its own copy of the array at its own address for the life of the
// process.  In host code the array's NAME is only a handle for hipGetSymbolAddress: kernels are
// given the per-device address obtained from it, never the name.
#define SP_STATIC_SCRATCH_BYTES_IMPL ((size_t)32 << 20)
static __device__ __align__(256) unsigned char scratch[SP_STATIC_SCRATCH_BYTES_IMPL];

namespace sp {
namespace { std::atomic<int> g_small_steps{-1}; }      // < 0: the rule of use_small_shape()
int small_shape_steps() { return g_small_steps.load(std::memory_order_relaxed); }
}  // namespace sp

namespace {

thread_local char g_err[512] = "";

sp_status fail(sp_status code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Every workspace starts with a tag block of TAG_BYTES; the segment table follows it.  The tag says
// whether the workspace holds a forward's reserve (the part of o that its rounding to bf16 dropped) and for
// which outputs; every call rewrites or re-validates it before it writes anything else, so a reserve
// that some other call may have overwritten is never trusted.
constexpr size_t TAG_BYTES = 256;
inline int* table_of(void* workspace) { return (int*)((char*)workspace + TAG_BYTES); }
inline bool misaligned(const void* p) { return ((uintptr_t)p & 15) != 0; }

// Bytes of the schedule region that follows the table: key_lo and row_hi per token, then the tile
// descriptors (sized by upper bounds on the tile counts, so that it depends on the totals alone).
struct SchedLayout { size_t key_lo, row_hi, tiles256, tiles128, bytes; };
SchedLayout sched_layout(int64_t total_tokens, int32_t n_groups) {
    SchedLayout s{};
    const size_t per_tok = align256((size_t)total_tokens * 4);
    const size_t b256 = align256(((size_t)total_tokens / 256 + (size_t)n_groups + 1) * sizeof(sp::TileDesc));
    const size_t b128 = align256(((size_t)total_tokens / 128 + (size_t)n_groups + 1) * sizeof(sp::TileDesc));
    s.key_lo = 0; s.row_hi = per_tok; s.tiles256 = 2 * per_tok; s.tiles128 = s.tiles256 + b256; s.bytes = s.tiles128 + b128;
    return s;
}

size_t table_words(int32_t n_groups, int64_t total_responses) {
    return (size_t)sp::TAB_HEADER + (size_t)sp::TAB_GROUP_WORDS * n_groups + (size_t)total_responses + n_groups;
}

sp_status check_geometry(int32_t Hq, int32_t Hkv, int32_t d, float scale, sp_dtype dtype) {
    if (Hq < 1 || Hkv < 1 || Hq % Hkv != 0)
        return fail(SP_ERR_INVALID_ARG, "n_q_heads=%d must be a positive multiple of n_kv_heads=%d", Hq, Hkv);
    if (!std::isfinite(scale) || scale <= 0.f)
        return fail(SP_ERR_INVALID_ARG, "softmax_scale must be finite and > 0");
    if (dtype == SP_BF16) {
        if (d != 128) return fail(SP_ERR_UNSUPPORTED, "bf16 path supports head_dim 128 only (got %d)", d);
    } else if (dtype == SP_F32) {
        if (d != 64 && d != 128) return fail(SP_ERR_UNSUPPORTED, "fp32 path supports head_dim 64 or 128 (got %d)", d);
    } else {
        return fail(SP_ERR_UNSUPPORTED, "unknown dtype %d", (int)dtype);
    }
    return SP_OK;
}

struct Layout {
    std::vector<int32_t> words;       // the segment table
    std::vector<int> group_tokens;
    int64_t total_tokens = 0;
    int64_t total_responses = 0;
    int max_group_tokens = 0;
    int min_prompt_len = 0x7fffffff;
};

sp_status build_table(int32_t n_groups, const int32_t* prompt_lens, const int32_t* Gs,
                      const int32_t* resp_lens_flat, Layout& L) {
    if (n_groups < 1) return fail(SP_ERR_INVALID_ARG, "n_groups must be >= 1");
    if (!prompt_lens || !Gs) return fail(SP_ERR_INVALID_ARG, "prompt_lens / Gs is NULL");
    int64_t nresp = 0;
    for (int g = 0; g < n_groups; ++g) {
        if (Gs[g] < 0) return fail(SP_ERR_INVALID_ARG, "group %d: G=%d is negative", g, Gs[g]);
        nresp += Gs[g];
    }
    if (nresp > 0 && !resp_lens_flat) return fail(SP_ERR_INVALID_ARG, "resp_lens is NULL but G > 0");
    if (nresp > (int64_t)1 << 28) return fail(SP_ERR_INVALID_ARG, "too many responses");
    L.total_responses = nresp;
    L.words.assign(table_words(n_groups, nresp), 0);
    L.group_tokens.resize(n_groups);
    int64_t tok = 0, r = 0, tiles256 = 0, tiles128 = 0;
    size_t roff = (size_t)sp::TAB_HEADER + (size_t)sp::TAB_GROUP_WORDS * n_groups;
    for (int g = 0; g < n_groups; ++g) {
        if (prompt_lens[g] < 0) return fail(SP_ERR_INVALID_ARG, "group %d: prompt_len is negative", g);
        if (prompt_lens[g] < L.min_prompt_len) L.min_prompt_len = prompt_lens[g];
        int64_t tg = prompt_lens[g];
        int32_t* e = &L.words[sp::TAB_HEADER + sp::TAB_GROUP_WORDS * g];
        e[0] = (int32_t)tok; e[1] = prompt_lens[g]; e[3] = (int32_t)roff; e[4] = Gs[g];
        e[sp::TAB_TILES256] = (int32_t)tiles256; e[sp::TAB_TILES128] = (int32_t)tiles128;
        L.words[roff++] = prompt_lens[g];
        for (int i = 0; i < Gs[g]; ++i, ++r) {
            if (resp_lens_flat[r] < 0) return fail(SP_ERR_INVALID_ARG, "group %d: response %d has negative length", g, i);
            tg += resp_lens_flat[r];
            if (tg > 0x7fff0000LL) return fail(SP_ERR_INVALID_ARG, "group %d holds too many tokens", g);
            L.words[roff++] = (int32_t)tg;
        }
        if (tg < 1) return fail(SP_ERR_INVALID_ARG, "group %d is empty (needs at least one token)", g);
        e[2] = (int32_t)tg;
        L.group_tokens[g] = (int)tg;
        if (tg > L.max_group_tokens) L.max_group_tokens = (int)tg;
        tok += tg;
        tiles256 += (tg + 255) / 256; tiles128 += (tg + 127) / 128;
        if (tok > 0x7fff0000LL) return fail(SP_ERR_INVALID_ARG, "total token count exceeds the int32 range");
    }
    L.total_tokens = tok;
    L.words[0] = n_groups; L.words[1] = (int32_t)tok; L.words[2] = (int32_t)L.words.size();
    return SP_OK;
}

sp_status run(bool bwd, const void* q, const void* k, const void* v, const void* o, const float* lse,
              const void* d_o, void* o_out, float* lse_out, void* dq, void* dk, void* dv,
              int32_t n_groups, const int32_t* prompt_lens, const int32_t* Gs, const int32_t* resp_lens_flat,
              int32_t Hq, int32_t Hkv, int32_t d, float scale, sp_dtype dtype, sp_schedule schedule,
              unsigned stages, unsigned flags, void* workspace, size_t workspace_bytes, void* stream,
              void* o_lo = nullptr) {
    g_err[0] = 0;
    if (o_lo && misaligned(o_lo)) return fail(SP_ERR_INVALID_ARG, "o_lo pointer %p is not 16-byte aligned", o_lo);
    if (o_lo && dtype != SP_BF16) return fail(SP_ERR_UNSUPPORTED, "o_lo is a bf16 option (fp32 outputs are not rounded)");
    if (flags & ~(unsigned)(SP_FLAG_RESPONSE_ROWS | SP_FLAG_ACCUMULATE_DKDV))
        return fail(SP_ERR_INVALID_ARG, "unknown bits in flags=0x%x", flags);
    if (!bwd && (flags & SP_FLAG_ACCUMULATE_DKDV))
        return fail(SP_ERR_INVALID_ARG, "SP_FLAG_ACCUMULATE_DKDV is a backward flag");
    sp_status st = check_geometry(Hq, Hkv, d, scale, dtype);
    if (st != SP_OK) return st;
    if (schedule != SP_SCHED_SHARED && schedule != SP_SCHED_NAIVE_CAUSAL)
        return fail(SP_ERR_INVALID_ARG, "unknown schedule %d", (int)schedule);
    if (bwd && (stages == 0 || (stages & ~(unsigned)SP_BWD_STAGE_ALL)))
        return fail(SP_ERR_INVALID_ARG, "stages=0x%x is not a non-empty subset of SP_BWD_STAGE_ALL", stages);
    const void* ptrs[] = {q, k, v, bwd ? o : o_out, bwd ? (const void*)lse : (const void*)lse_out,
                          bwd ? d_o : q, bwd ? dq : q, bwd ? dk : q, bwd ? dv : q};
    for (const void* p : ptrs) {
        if (!p) return fail(SP_ERR_INVALID_ARG, "a tensor pointer is NULL");
        if (misaligned(p)) return fail(SP_ERR_INVALID_ARG, "tensor pointer %p is not 16-byte aligned", p);
    }
    Layout L;
    st = build_table(n_groups, prompt_lens, Gs, resp_lens_flat, L);
    if (st != SP_OK) return st;
    const size_t need = sp_attn_workspace_bytes(bwd, L.total_tokens, n_groups, L.total_responses, Hq, Hkv, d, dtype);
    if (!workspace || misaligned(workspace) || workspace_bytes < need)
        return fail(SP_ERR_WORKSPACE, "workspace %p of %zu bytes; need %zu bytes, 16-byte aligned", workspace,
                    workspace_bytes, need);

    // The reserve sits behind everything a backward of this problem keeps in the workspace, so the
    // forward and its backward find it at the same offset.
    const size_t reserve_off = align256(sp_attn_workspace_bytes(1, L.total_tokens, n_groups, L.total_responses, Hq, Hkv, d, dtype));
    const size_t reserve_len = sp_attn_reserve_bytes(L.total_tokens, Hq, d, dtype);
    const bool reserve_fits = reserve_len > 0 && workspace_bytes >= reserve_off + reserve_len;
    void* const reserve = (char*)workspace + reserve_off;
    const bool resp_only = (flags & SP_FLAG_RESPONSE_ROWS) != 0;
    sp::ReserveTag tag{};
    int tag_mode = sp::TAG_CLEAR;
    if (reserve_fits && !o_lo && !(bwd == false && schedule == SP_SCHED_NAIVE_CAUSAL)) {
        const uint64_t po = (uint64_t)(uintptr_t)(bwd ? o : o_out), pl = (uint64_t)(uintptr_t)(bwd ? (const void*)lse : (const void*)lse_out);
        tag.w[0] = sp::TAG_MAGIC;
        tag.w[1] = (uint32_t)po; tag.w[2] = (uint32_t)(po >> 32);
        tag.w[3] = (uint32_t)pl; tag.w[4] = (uint32_t)(pl >> 32);
        tag.w[5] = (uint32_t)L.total_tokens; tag.w[6] = (uint32_t)Hq; tag.w[7] = (uint32_t)d;
        tag.w[8] = (uint32_t)reserve_off; tag.w[9] = (uint32_t)((uint64_t)reserve_off >> 32);
        tag.w[10] = resp_only ? 1u : 0u;        // a reserve written for response rows only serves only such a backward
        tag_mode = bwd ? sp::TAG_CHECK : sp::TAG_WRITE;
    }
    // gradient stages enqueued on their own run on the workspace that their ROWSUM stage prepared (and
    // checked): the tag is left as it is
    const bool keep_tag = bwd && !(stages & SP_BWD_STAGE_ROWSUM);

    hipStream_t s = (hipStream_t)stream;
    sp::Problem p{};
    p.q = q; p.k = k; p.v = v; p.o = o; p.lse = lse; p.d_o = d_o;
    p.o_out = o_out; p.lse_out = lse_out; p.dq = dq; p.dk = dk; p.dv = dv;
    p.tab = table_of(workspace);
    char* const sched_base = (char*)workspace + TAG_BYTES + align256(L.words.size() * 4);
    const SchedLayout sl = sched_layout(L.total_tokens, n_groups);
    p.sched = sp::Schedule{(const sp::TileDesc*)(sched_base + sl.tiles256), (const sp::TileDesc*)(sched_base + sl.tiles128),
                           (const int*)(sched_base + sl.key_lo), (const int*)(sched_base + sl.row_hi)};
    p.Dbuf = (float*)(sched_base + sl.bytes);
    p.dkdv_partial = (bwd && dtype == SP_BF16 && sp::dkdv_head_split(L.total_tokens, n_groups, Hq, Hkv))
                         ? (float*)((char*)p.Dbuf + align256((size_t)Hq * (size_t)L.total_tokens * 8)) : nullptr;
    p.n_groups = n_groups; p.total_tokens = L.total_tokens; p.max_group_tokens = L.max_group_tokens;
    p.total_responses = L.total_responses; p.min_prompt_len = L.min_prompt_len;
    p.Hq = Hq; p.Hkv = Hkv; p.head_dim = d; p.scale = scale;
    p.naive = schedule == SP_SCHED_NAIVE_CAUSAL;
    p.stages = stages;
    p.resp_only = resp_only;
    // rounding residual of o: the caller's tensor if given, else the workspace's reserve (forward: written
    // when the workspace has room for it; backward: used if the tag check on the device finds it valid)
    p.o_lo_out = bwd ? nullptr : (o_lo ? o_lo : (tag_mode == sp::TAG_WRITE ? reserve : nullptr));
    p.o_lo = bwd ? (o_lo ? o_lo : (tag_mode == sp::TAG_CHECK ? reserve : nullptr)) : nullptr;
    p.o_lo_flag = (bwd && !o_lo && tag_mode == sp::TAG_CHECK) ? (const uint32_t*)workspace + sp::TAG_FLAG_WORD : nullptr;
    p.accumulate = (flags & SP_FLAG_ACCUMULATE_DKDV) != 0;
    p.host_group_tokens = L.group_tokens.data();
    p.host_table = L.words.data();

    p.n_tiles256 = sp::count_tiles(p, 256); p.n_tiles128 = sp::count_tiles(p, 128);
    hipError_t e = sp::launch_prepare(L.words.data(), (int)L.words.size(), table_of(workspace), (uint32_t*)workspace, tag,
                                      keep_tag ? sp::TAG_KEEP : tag_mode, dtype == SP_BF16, n_groups, L.total_tokens,
                                      p.n_tiles256, p.n_tiles128, p.sched, s);
    if (e == hipSuccess) {
        if (dtype == SP_BF16) e = bwd ? sp::launch_bwd_bf16(p, s) : sp::launch_fwd_bf16(p, s);
        else e = bwd ? sp::launch_bwd_f32(p, s) : sp::launch_fwd_f32(p, s);
    }
    if (e != hipSuccess) return fail(SP_ERR_DEVICE, "HIP launch failed: %s", hipGetErrorString(e));
    return SP_OK;
}

}  // namespace

extern "C" {

size_t sp_attn_workspace_bytes(int is_bwd, int64_t total_tokens, int32_t n_groups, int64_t total_responses,
                               int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, sp_dtype dtype) {
    (void)head_dim;
    if (total_tokens < 1 || n_groups < 1 || total_responses < 0 || n_q_heads < 1) return 0;
    size_t bytes = TAG_BYTES + align256(table_words(n_groups, total_responses) * 4) + sched_layout(total_tokens, n_groups).bytes;
    if (is_bwd) bytes += align256((size_t)n_q_heads * (size_t)total_tokens * 8);   // D and scaled LSE
    if (is_bwd && dtype == SP_BF16 && n_kv_heads > 0 && n_q_heads % n_kv_heads == 0 &&
        sp::dkdv_head_split(total_tokens, n_groups, n_q_heads, n_kv_heads))       // per-q-head dK, dV partials
        bytes += align256((size_t)2 * (n_q_heads / n_kv_heads) * (size_t)total_tokens * n_kv_heads * 128 * 4);
    return bytes;
}

size_t sp_attn_reserve_bytes(int64_t total_tokens, int32_t n_q_heads, int32_t head_dim, sp_dtype dtype) {
    if (total_tokens < 1 || n_q_heads < 1 || head_dim < 1 || dtype != SP_BF16) return 0;
    return align256((size_t)total_tokens * (size_t)n_q_heads * (size_t)head_dim * 2);
}

sp_status sp_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse, int32_t prompt_len,
                      const int32_t* resp_lens, int32_t G, int32_t n_q_heads, int32_t n_kv_heads,
                      int32_t head_dim, float softmax_scale, sp_dtype dtype, void* workspace,
                      size_t workspace_bytes, void* stream) {
    return run(false, q, k, v, nullptr, nullptr, nullptr, o, lse, nullptr, nullptr, nullptr, 1, &prompt_len, &G,
               resp_lens, n_q_heads, n_kv_heads, head_dim, softmax_scale, dtype, SP_SCHED_SHARED, SP_BWD_STAGE_ALL, 0u, workspace,
               workspace_bytes, stream);
}

sp_status sp_attn_bwd(const void* q, const void* k, const void* v, const void* o, const float* lse,
                      const void* d_o, void* dq, void* dk, void* dv, int32_t prompt_len, const int32_t* resp_lens,
                      int32_t G, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, float softmax_scale,
                      sp_dtype dtype, void* workspace, size_t workspace_bytes, void* stream) {
    return run(true, q, k, v, o, lse, d_o, nullptr, nullptr, dq, dk, dv, 1, &prompt_len, &G, resp_lens, n_q_heads,
               n_kv_heads, head_dim, softmax_scale, dtype, SP_SCHED_SHARED, SP_BWD_STAGE_ALL, 0u, workspace, workspace_bytes, stream);
}

sp_status sp_attn_fwd_batched(const void* q, const void* k, const void* v, void* o, float* lse, int32_t n_groups,
                              const int32_t* prompt_lens, const int32_t* Gs, const int32_t* resp_lens_flat,
                              int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, float softmax_scale,
                              sp_dtype dtype, sp_schedule schedule, void* workspace, size_t workspace_bytes,
                              void* stream) {
    return run(false, q, k, v, nullptr, nullptr, nullptr, o, lse, nullptr, nullptr, nullptr, n_groups, prompt_lens,
               Gs, resp_lens_flat, n_q_heads, n_kv_heads, head_dim, softmax_scale, dtype, schedule, SP_BWD_STAGE_ALL, 0u, workspace,
               workspace_bytes, stream);
}

sp_status sp_attn_bwd_batched(const void* q, const void* k, const void* v, const void* o, const float* lse,
                              const void* d_o, void* dq, void* dk, void* dv, int32_t n_groups,
                              const int32_t* prompt_lens, const int32_t* Gs, const int32_t* resp_lens_flat,
                              int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, float softmax_scale,
                              sp_dtype dtype, void* workspace, size_t workspace_bytes, void* stream) {
    return run(true, q, k, v, o, lse, d_o, nullptr, nullptr, dq, dk, dv, n_groups, prompt_lens, Gs, resp_lens_flat,
               n_q_heads, n_kv_heads, head_dim, softmax_scale, dtype, SP_SCHED_SHARED, SP_BWD_STAGE_ALL, 0u, workspace, workspace_bytes,
               stream);
}

sp_status sp_attn_bwd_batched_stages(const void* q, const void* k, const void* v, const void* o, const float* lse,
                                     const void* d_o, void* dq, void* dk, void* dv, int32_t n_groups,
                                     const int32_t* prompt_lens, const int32_t* Gs, const int32_t* resp_lens_flat,
                                     int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, float softmax_scale,
                                     sp_dtype dtype, uint32_t stages, void* workspace, size_t workspace_bytes,
                                     void* stream) {
    // outputs of stages that do not run may be NULL: substitute q so the pointer checks pass
    if (!(stages & SP_BWD_STAGE_ROWSUM) && !o) o = q;
    if (!(stages & SP_BWD_STAGE_DQ) && !dq) dq = const_cast<void*>(q);
    if (!(stages & SP_BWD_STAGE_DKDV)) { if (!dk) dk = const_cast<void*>(q); if (!dv) dv = const_cast<void*>(q); }
    return run(true, q, k, v, o, lse, d_o, nullptr, nullptr, dq, dk, dv, n_groups, prompt_lens, Gs, resp_lens_flat,
               n_q_heads, n_kv_heads, head_dim, softmax_scale, dtype, SP_SCHED_SHARED, stages, 0u, workspace,
               workspace_bytes, stream);
}

sp_status sp_attn_fwd_batched_ex(const void* q, const void* k, const void* v, void* o, float* lse, int32_t n_groups,
                                 const int32_t* prompt_lens, const int32_t* Gs, const int32_t* resp_lens_flat,
                                 int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, float softmax_scale,
                                 sp_dtype dtype, sp_schedule schedule, uint32_t flags, void* o_lo, void* workspace,
                                 size_t workspace_bytes, void* stream) {
    return run(false, q, k, v, nullptr, nullptr, nullptr, o, lse, nullptr, nullptr, nullptr, n_groups, prompt_lens,
               Gs, resp_lens_flat, n_q_heads, n_kv_heads, head_dim, softmax_scale, dtype, schedule, SP_BWD_STAGE_ALL,
               flags, workspace, workspace_bytes, stream, o_lo);
}

sp_status sp_attn_bwd_batched_ex(const void* q, const void* k, const void* v, const void* o, const float* lse,
                                 const void* d_o, void* dq, void* dk, void* dv, int32_t n_groups,
                                 const int32_t* prompt_lens, const int32_t* Gs, const int32_t* resp_lens_flat,
                                 int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, float softmax_scale,
                                 sp_dtype dtype, uint32_t stages, uint32_t flags, const void* o_lo,
                                 void* workspace, size_t workspace_bytes, void* stream) {
    if (!(stages & SP_BWD_STAGE_ROWSUM) && !o) o = q;
    if (!(stages & SP_BWD_STAGE_DQ) && !dq) dq = const_cast<void*>(q);
    if (!(stages & SP_BWD_STAGE_DKDV)) { if (!dk) dk = const_cast<void*>(q); if (!dv) dv = const_cast<void*>(q); }
    return run(true, q, k, v, o, lse, d_o, nullptr, nullptr, dq, dk, dv, n_groups, prompt_lens, Gs, resp_lens_flat,
               n_q_heads, n_kv_heads, head_dim, softmax_scale, dtype, SP_SCHED_SHARED, stages, flags, workspace,
               workspace_bytes, stream, const_cast<void*>(o_lo));
}

sp_status sp_attn_fwd_multi(int32_t n_sets, const void* const* q, const void* const* k, const void* const* v,
                            void* const* o, float* const* lse, int32_t n_groups, const int32_t* prompt_lens,
                            const int32_t* Gs, const int32_t* resp_lens_flat, int32_t n_q_heads, int32_t n_kv_heads,
                            int32_t head_dim, float softmax_scale, sp_dtype dtype, void* workspace,
                            size_t workspace_bytes, void* stream) {
    g_err[0] = 0;
    if (n_sets < 1 || n_sets > SP_MAX_SETS)
        return fail(SP_ERR_INVALID_ARG, "n_sets=%d is outside 1..%d", n_sets, SP_MAX_SETS);
    if (!q || !k || !v || !o || !lse) return fail(SP_ERR_INVALID_ARG, "a pointer array is NULL");
    sp_status st = check_geometry(n_q_heads, n_kv_heads, head_dim, softmax_scale, dtype);
    if (st != SP_OK) return st;
    for (int i = 0; i < n_sets; ++i) {
        const void* ptrs[] = {q[i], k[i], v[i], o[i], lse[i]};
        for (const void* p : ptrs) {
            if (!p) return fail(SP_ERR_INVALID_ARG, "set %d: a tensor pointer is NULL", i);
            if (misaligned(p)) return fail(SP_ERR_INVALID_ARG, "set %d: tensor pointer %p is not 16-byte aligned", i, p);
        }
    }
    Layout L;
    st = build_table(n_groups, prompt_lens, Gs, resp_lens_flat, L);
    if (st != SP_OK) return st;
    const size_t need = sp_attn_workspace_bytes(0, L.total_tokens, n_groups, L.total_responses, n_q_heads, n_kv_heads,
                                                head_dim, dtype);
    if (!workspace || misaligned(workspace) || workspace_bytes < need)
        return fail(SP_ERR_WORKSPACE, "workspace %p of %zu bytes; need %zu bytes, 16-byte aligned", workspace,
                    workspace_bytes, need);
    hipStream_t s = (hipStream_t)stream;
    sp::Problem p{};
    p.tab = table_of(workspace);
    p.n_groups = n_groups; p.total_tokens = L.total_tokens; p.max_group_tokens = L.max_group_tokens;
    p.total_responses = L.total_responses; p.min_prompt_len = L.min_prompt_len;
    p.Hq = n_q_heads; p.Hkv = n_kv_heads; p.head_dim = head_dim; p.scale = softmax_scale;
    p.host_group_tokens = L.group_tokens.data();
    p.host_table = L.words.data();
    char* const sched_base = (char*)workspace + TAG_BYTES + align256(L.words.size() * 4);
    const SchedLayout sl = sched_layout(L.total_tokens, n_groups);
    p.sched = sp::Schedule{(const sp::TileDesc*)(sched_base + sl.tiles256), (const sp::TileDesc*)(sched_base + sl.tiles128),
                           (const int*)(sched_base + sl.key_lo), (const int*)(sched_base + sl.row_hi)};
    p.n_tiles256 = sp::count_tiles(p, 256); p.n_tiles128 = sp::count_tiles(p, 128);
    hipError_t e = sp::launch_prepare(L.words.data(), (int)L.words.size(), table_of(workspace), (uint32_t*)workspace,
                                      sp::ReserveTag{}, sp::TAG_CLEAR, dtype == SP_BF16, n_groups, L.total_tokens,
                                      p.n_tiles256, p.n_tiles128, p.sched, s);
    if (e == hipSuccess) {
        if (dtype == SP_BF16) {
            p.n_sets = n_sets;
            for (int i = 0; i < n_sets; ++i) { p.qs[i] = q[i]; p.ks[i] = k[i]; p.vs[i] = v[i]; p.os[i] = o[i]; p.lses[i] = lse[i]; }
            if (n_sets == 1) { p.q = q[0]; p.k = k[0]; p.v = v[0]; p.o_out = o[0]; p.lse_out = lse[0]; }
            e = sp::launch_fwd_bf16(p, s);
        } else {                 // the fp32 debug kernels take one set per launch
            for (int i = 0; i < n_sets && e == hipSuccess; ++i) {
                p.q = q[i]; p.k = k[i]; p.v = v[i]; p.o_out = o[i]; p.lse_out = lse[i];
                e = sp::launch_fwd_f32(p, s);
            }
        }
    }
    if (e != hipSuccess) return fail(SP_ERR_DEVICE, "HIP launch failed: %s", hipGetErrorString(e));
    return SP_OK;
}

namespace {
sp_status rope_call(const void* x, void* y, int32_t H, const void* x2, void* y2, int32_t H2, int32_t inverse,
                    int32_t n_groups, const int32_t* prompt_lens, const int32_t* Gs, const int32_t* resp_lens_flat,
                    int32_t head_dim, double rope_base, sp_dtype dtype, void* workspace, size_t workspace_bytes,
                    void* stream) {
    g_err[0] = 0;
    if (!x || !y || (x2 && !y2)) return fail(SP_ERR_INVALID_ARG, "a tensor pointer is NULL");
    if (misaligned(x) || misaligned(y) || misaligned(x2) || misaligned(y2))
        return fail(SP_ERR_INVALID_ARG, "tensor pointer is not 16-byte aligned");
    if (H < 1 || (x2 && H2 < 1)) return fail(SP_ERR_INVALID_ARG, "head counts %d, %d", H, H2);
    if (!(rope_base > 1.0) || !std::isfinite(rope_base))
        return fail(SP_ERR_INVALID_ARG, "rope_base must be finite and > 1");
    if (dtype != SP_BF16 && dtype != SP_F32) return fail(SP_ERR_UNSUPPORTED, "unknown dtype %d", (int)dtype);
    if (head_dim != 64 && head_dim != 128) return fail(SP_ERR_UNSUPPORTED, "head_dim=%d (64 or 128)", head_dim);
    Layout L;
    sp_status st = build_table(n_groups, prompt_lens, Gs, resp_lens_flat, L);
    if (st != SP_OK) return st;
    const size_t need = sp_attn_workspace_bytes(0, L.total_tokens, n_groups, L.total_responses, H, H, head_dim, dtype);
    if (!workspace || misaligned(workspace) || workspace_bytes < need)
        return fail(SP_ERR_WORKSPACE, "workspace %p of %zu bytes; need %zu bytes, 16-byte aligned", workspace,
                    workspace_bytes, need);
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = sp::launch_prepare(L.words.data(), (int)L.words.size(), table_of(workspace), (uint32_t*)workspace,
                                      sp::ReserveTag{}, sp::TAG_CLEAR, false, n_groups, L.total_tokens, 0, 0, sp::Schedule{}, s);
    if (e == hipSuccess)
        e = sp::launch_rope(x, y, H, x2, y2, H2, table_of(workspace), L.total_tokens, head_dim, rope_base, inverse != 0,
                            dtype == SP_F32, s);
    if (e != hipSuccess) return fail(SP_ERR_DEVICE, "HIP launch failed: %s", hipGetErrorString(e));
    return SP_OK;
}
}  // namespace

sp_status sp_attn_rope(const void* x, void* y, int32_t n_heads, int32_t inverse, int32_t n_groups,
                       const int32_t* prompt_lens, const int32_t* Gs, const int32_t* resp_lens_flat,
                       int32_t head_dim, double rope_base, sp_dtype dtype, void* workspace, size_t workspace_bytes,
                       void* stream) {
    return rope_call(x, y, n_heads, nullptr, nullptr, 0, inverse, n_groups, prompt_lens, Gs, resp_lens_flat, head_dim,
                     rope_base, dtype, workspace, workspace_bytes, stream);
}

sp_status sp_attn_rope_qk(const void* q, void* q_out, int32_t n_q_heads, const void* k, void* k_out, int32_t n_kv_heads,
                          int32_t inverse, int32_t n_groups, const int32_t* prompt_lens, const int32_t* Gs,
                          const int32_t* resp_lens_flat, int32_t head_dim, double rope_base, sp_dtype dtype,
                          void* workspace, size_t workspace_bytes, void* stream) {
    if (!k || !k_out) { g_err[0] = 0; return fail(SP_ERR_INVALID_ARG, "a tensor pointer is NULL"); }
    return rope_call(q, q_out, n_q_heads, k, k_out, n_kv_heads, inverse, n_groups, prompt_lens, Gs, resp_lens_flat,
                     head_dim, rope_base, dtype, workspace, workspace_bytes, stream);
}

size_t sp_attn_loss_workspace_bytes(int64_t total_tokens, int32_t n_groups, int64_t total_responses) {
    if (total_tokens < 1 || n_groups < 1 || total_responses < 0) return 0;
    return TAG_BYTES + align256(table_words(n_groups, total_responses) * 4) + align256((size_t)(total_responses + 1) * 4);
}

namespace {
// shared front end of the three loss calls: packing -> table in the workspace
sp_status loss_setup(int32_t n_groups, const int32_t* prompt_lens, const int32_t* Gs, const int32_t* resp_lens_flat,
                     void* workspace, size_t workspace_bytes, hipStream_t s, Layout& L, float** scratch) {
    sp_status st = build_table(n_groups, prompt_lens, Gs, resp_lens_flat, L);
    if (st != SP_OK) return st;
    const size_t need = sp_attn_loss_workspace_bytes(L.total_tokens, n_groups, L.total_responses);
    if (!workspace || misaligned(workspace) || workspace_bytes < need)
        return fail(SP_ERR_WORKSPACE, "workspace %p of %zu bytes; need %zu bytes, 16-byte aligned", workspace,
                    workspace_bytes, need);
    *scratch = (float*)((char*)workspace + TAG_BYTES + align256(L.words.size() * 4));
    hipError_t e = sp::launch_prepare(L.words.data(), (int)L.words.size(), table_of(workspace), (uint32_t*)workspace,
                                      sp::ReserveTag{}, sp::TAG_CLEAR, false, n_groups, L.total_tokens, 0, 0, sp::Schedule{}, s);
    if (e != hipSuccess) return fail(SP_ERR_DEVICE, "HIP launch failed: %s", hipGetErrorString(e));
    return SP_OK;
}
}  // namespace

sp_status sp_attn_logprob_fwd(const void* logits, const int32_t* labels, float* logp, float* lse, int64_t vocab,
                              int32_t n_groups, const int32_t* prompt_lens, const int32_t* Gs,
                              const int32_t* resp_lens_flat, sp_dtype dtype, void* workspace, size_t workspace_bytes,
                              void* stream) {
    g_err[0] = 0;
    if (!logits || !labels || !logp || !lse) return fail(SP_ERR_INVALID_ARG, "a pointer is NULL");
    if (misaligned(logits)) return fail(SP_ERR_INVALID_ARG, "logits pointer is not 16-byte aligned");
    if (vocab < 1) return fail(SP_ERR_INVALID_ARG, "vocab=%lld", (long long)vocab);
    if (dtype != SP_BF16 && dtype != SP_F32) return fail(SP_ERR_UNSUPPORTED, "unknown dtype %d", (int)dtype);
    Layout L; float* scratch = nullptr;
    sp_status st = loss_setup(n_groups, prompt_lens, Gs, resp_lens_flat, workspace, workspace_bytes, (hipStream_t)stream, L, &scratch);
    if (st != SP_OK) return st;
    hipError_t e = sp::launch_logprob_fwd(logits, labels, logp, lse, table_of(workspace), L.total_tokens, vocab,
                                          dtype == SP_F32, (hipStream_t)stream);
    if (e != hipSuccess) return fail(SP_ERR_DEVICE, "HIP launch failed: %s", hipGetErrorString(e));
    return SP_OK;
}

sp_status sp_attn_logprob_bwd(const void* logits, const int32_t* labels, const float* lse, const float* g,
                              void* dlogits, int64_t vocab, int32_t n_groups, const int32_t* prompt_lens,
                              const int32_t* Gs, const int32_t* resp_lens_flat, sp_dtype dtype, void* workspace,
                              size_t workspace_bytes, void* stream) {
    g_err[0] = 0;
    if (!logits || !labels || !lse || !g || !dlogits) return fail(SP_ERR_INVALID_ARG, "a pointer is NULL");
    if (misaligned(logits) || misaligned(dlogits)) return fail(SP_ERR_INVALID_ARG, "tensor pointer is not 16-byte aligned");
    if (vocab < 1) return fail(SP_ERR_INVALID_ARG, "vocab=%lld", (long long)vocab);
    if (dtype != SP_BF16 && dtype != SP_F32) return fail(SP_ERR_UNSUPPORTED, "unknown dtype %d", (int)dtype);
    Layout L; float* scratch = nullptr;
    sp_status st = loss_setup(n_groups, prompt_lens, Gs, resp_lens_flat, workspace, workspace_bytes, (hipStream_t)stream, L, &scratch);
    if (st != SP_OK) return st;
    hipError_t e = sp::launch_logprob_bwd(logits, labels, lse, g, dlogits, table_of(workspace), L.total_tokens, vocab,
                                          dtype == SP_F32, (hipStream_t)stream);
    if (e != hipSuccess) return fail(SP_ERR_DEVICE, "HIP launch failed: %s", hipGetErrorString(e));
    return SP_OK;
}

sp_status sp_attn_grpo_loss(const float* logp, const float* logp_old, const float* logp_ref, const float* adv,
                            float eps_low, float eps_high, float beta, float* loss, float* g, int32_t n_groups,
                            const int32_t* prompt_lens, const int32_t* Gs, const int32_t* resp_lens_flat,
                            void* workspace, size_t workspace_bytes, void* stream) {
    g_err[0] = 0;
    if (!logp || !logp_old || !logp_ref || !adv || !loss || !g) return fail(SP_ERR_INVALID_ARG, "a pointer is NULL");
    if (!(eps_low >= 0.f && eps_low < 1.f) || !(eps_high >= 0.f) || !std::isfinite(eps_high) || !std::isfinite(beta))
        return fail(SP_ERR_INVALID_ARG, "eps_low must lie in [0, 1), eps_high in [0, inf), beta finite");
    Layout L; float* scratch = nullptr;
    sp_status st = loss_setup(n_groups, prompt_lens, Gs, resp_lens_flat, workspace, workspace_bytes, (hipStream_t)stream, L, &scratch);
    if (st != SP_OK) return st;
    int nonempty = 0;
    for (int64_t r = 0; r < L.total_responses; ++r) nonempty += resp_lens_flat[r] > 0;
    hipError_t e = sp::launch_grpo(logp, logp_old, logp_ref, adv, g, scratch, loss, table_of(workspace),
                                   (int)L.total_responses, nonempty, eps_low, eps_high, beta, (hipStream_t)stream);
    if (e != hipSuccess) return fail(SP_ERR_DEVICE, "HIP launch failed: %s", hipGetErrorString(e));
    return SP_OK;
}

sp_status sp_attn_segment_table(int32_t n_groups, const int32_t* prompt_lens, const int32_t* Gs,
                                const int32_t* resp_lens_flat, int32_t* words, size_t capacity,
                                size_t* n_words) {
    g_err[0] = 0;
    if (!n_words) return fail(SP_ERR_INVALID_ARG, "n_words is NULL");
    Layout L;
    sp_status st = build_table(n_groups, prompt_lens, Gs, resp_lens_flat, L);
    if (st != SP_OK) return st;
    *n_words = L.words.size();
    if (!words || capacity < L.words.size())
        return fail(SP_ERR_WORKSPACE, "segment table needs %zu words, capacity is %zu", L.words.size(), words ? capacity : (size_t)0);
    for (size_t i = 0; i < L.words.size(); ++i) words[i] = L.words[i];
    return SP_OK;
}

sp_status sp_attn_row_tile(int32_t n_groups, const int32_t* prompt_lens, const int32_t* Gs,
                           const int32_t* resp_lens_flat, int32_t* rows, int64_t* steps_256, int64_t* steps_128) {
    g_err[0] = 0;
    if (!rows) return fail(SP_ERR_INVALID_ARG, "rows is NULL");
    Layout L;
    sp_status st = build_table(n_groups, prompt_lens, Gs, resp_lens_flat, L);
    if (st != SP_OK) return st;
    sp::Problem p{};
    p.n_groups = n_groups;
    p.host_table = L.words.data();
    int64_t s256, t256, s128, t128;
    sp::key_steps(p, 256, s256, t256);
    sp::key_steps(p, 128, s128, t128);
    *rows = sp::use_small_shape(p) ? 128 : 256;
    if (steps_256) *steps_256 = s256;
    if (steps_128) *steps_128 = s128;
    return SP_OK;
}

namespace {
constexpr int MAX_DEVICES = 64;
std::atomic<void*> g_scratch_ptr[MAX_DEVICES];      // device address of `scratch` on each GPU, 0 = not asked yet
}

sp_status sp_attn_bwd_batched_static(const void* q, const void* k, const void* v, const void* o, const float* lse,
                                     const void* d_o, void* dq, void* dk, void* dv, int32_t n_groups,
                                     const int32_t* prompt_lens, const int32_t* Gs, const int32_t* resp_lens_flat,
                                     int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, float softmax_scale,
                                     sp_dtype dtype, void* stream) {
    static_assert(SP_STATIC_SCRATCH_BYTES_IMPL == SP_STATIC_SCRATCH_BYTES, "header and array disagree");
    g_err[0] = 0;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(SP_ERR_DEVICE, "hipGetDevice failed: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(SP_ERR_UNSUPPORTED, "device ordinal %d is outside 0..%d", dev, MAX_DEVICES - 1);
    void* ws = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ws) {
        // once per device, with that device current: each GPU has the array at its own address
        e = hipGetSymbolAddress(&ws, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ws)
            return fail(SP_ERR_DEVICE, "hipGetSymbolAddress(scratch) failed on device %d: %s", dev, hipGetErrorString(e));
        g_scratch_ptr[dev].store(ws, std::memory_order_release);
    }
    // Everything the kernels read from the scratch is written earlier in the same call (table by the
    // upload, D / scaled LSE by the rowsum stage, partial sums by the dkdv pass for every key), so
    // nothing has to be cleared; a problem that needs more than the array is rejected by the
    // workspace check of the common path before anything is enqueued.
    sp_status st = run(true, q, k, v, o, lse, d_o, nullptr, nullptr, dq, dk, dv, n_groups, prompt_lens, Gs,
                       resp_lens_flat, n_q_heads, n_kv_heads, head_dim, softmax_scale, dtype, SP_SCHED_SHARED,
                       SP_BWD_STAGE_ALL, 0u, ws, SP_STATIC_SCRATCH_BYTES, stream);
    if (st == SP_ERR_WORKSPACE) {
        char msg[sizeof(g_err)];
        snprintf(msg, sizeof(msg), "%s", g_err);
        return fail(SP_ERR_WORKSPACE, "problem exceeds the built-in scratch of %zu bytes (use sp_attn_bwd_batched "
                    "with a workspace): %.300s", (size_t)SP_STATIC_SCRATCH_BYTES, msg);
    }
    return st;
}

void sp_attn_set_small_shape_steps(int32_t steps) {
    sp::g_small_steps.store(steps < 0 ? -1 : steps, std::memory_order_relaxed);
}

const char* sp_attn_last_error(void) { return g_err; }
const char* sp_attn_version(void) { return "0.1"; }

}  // extern "C"
