// Internal launcher interface between the C-ABI layer (sp_api.hip) and the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "sp_common.hpp"

namespace sp {

constexpr unsigned STAGE_ROWSUM = 1u, STAGE_DKDV = 2u, STAGE_DQ = 4u;
constexpr int MAX_SETS = 4;      // tensor sets that one forward launch can serve

// Tag block at the head of every workspace (64 words).  Words 0..TAG_WORDS-1 describe the reserve a
// forward left in this workspace (magic, o and lse pointers, token count, heads, head_dim, byte offset of
// the reserve, response-rows-only flag); word TAG_FLAG_WORD is the verdict of the latest check.
constexpr int TAG_WORDS = 12;
constexpr int TAG_FLAG_WORD = 15;
constexpr uint32_t TAG_MAGIC = 0x53504152u;
struct ReserveTag { uint32_t w[TAG_WORDS]; };
// TAG_CLEAR: the workspace holds no reserve from here on.  TAG_WRITE: a forward is about to write the
// reserve that `tag` describes.  TAG_CHECK: a backward asks whether the workspace holds exactly the
// reserve `tag` describes; if not, the tag is cleared (the call is about to write into the workspace).
constexpr int TAG_CLEAR = 0, TAG_WRITE = 1, TAG_CHECK = 2;
constexpr int TAG_KEEP = -1;      // for launch_prepare: leave the tag block as it is

struct Problem {
    const void* q; const void* k; const void* v;
    const void* o; const float* lse; const void* d_o;     // backward inputs (o also fwd output)
    void* o_out; float* lse_out;                          // forward outputs
    // forward over several tensor sets that share one packing (n_sets > 1): set i reads qs/ks/vs[i]
    // and writes os/lses[i]; with n_sets <= 1 the single-set fields above are used
    int n_sets;
    const void* qs[MAX_SETS]; const void* ks[MAX_SETS]; const void* vs[MAX_SETS];
    void* os[MAX_SETS]; float* lses[MAX_SETS];
    void* dq; void* dk; void* dv;                         // backward outputs
    const int* tab;                                       // segment table (device)
    Schedule sched;                                       // tile descriptors and per-token segment bounds (device)
    int n_tiles256, n_tiles128;                           // exact tile counts of the packing
    float* Dbuf;                                          // [Hq, T_total] rowsum(dO*O) (device)
    int n_groups;
    int64_t total_tokens;
    int64_t total_responses;
    int min_prompt_len;                                   // shortest prompt of the batch
    int max_group_tokens;
    int Hq, Hkv, head_dim;
    float scale;
    int naive;                                            // forward: naive packed-causal schedule
    unsigned stages;                                      // backward: SP_BWD_STAGE_* bits to run
    int resp_only;                                        // only response rows are computed / contribute
    void* o_lo_out;                                       // forward (bf16): optional rounding residual of o
    const void* o_lo;                                     // backward (bf16): optional residual for D
    const uint32_t* o_lo_flag;                            // device word: o_lo may be used only if it is non-zero (NULL: always)
    int accumulate;                                       // backward: dk, dv += instead of =
    float* dkdv_partial;                                  // bf16 backward on small problems: fp32 per-q-head partials
    // host copies of the per-group token counts and of the whole segment table, for grid sizing and
    // for choosing kernel shapes
    const int* host_group_tokens;
    const int32_t* host_table;
};

hipError_t launch_fwd_bf16(const Problem& p, hipStream_t s);
hipError_t launch_bwd_bf16(const Problem& p, hipStream_t s);
hipError_t launch_fwd_f32(const Problem& p, hipStream_t s);
hipError_t launch_bwd_f32(const Problem& p, hipStream_t s);
hipError_t launch_rowsum(const Problem& p, bool f32, hipStream_t s);
// Rows that see at most EDGE_LEN keys are recomputed by the edge kernel (sp_edge.hip): D, and dQ, which
// the dq pass then does not store.
constexpr int EDGE_LEN = 64;
hipError_t launch_short_rows(const Problem& p, bool with_dq, hipStream_t s);
hipError_t launch_rope(const void* x, void* y, int H, const void* x2, void* y2, int H2, const int* tab,
                       int64_t total_tokens, int d, double base, bool inverse, bool f32, hipStream_t s);
hipError_t launch_logprob_fwd(const void* z, const int* y, float* logp, float* lse, const int* tab,
                              int64_t total_tokens, int64_t V, bool f32, hipStream_t s);
hipError_t launch_logprob_bwd(const void* z, const int* y, const float* lse, const float* g, void* dz,
                              const int* tab, int64_t total_tokens, int64_t V, bool f32, hipStream_t s);
hipError_t launch_grpo(const float* logp, const float* old, const float* ref, const float* adv, float* g,
                       float* J, float* loss, const int* tab, int n_resp, int n_nonempty, float eps_low,
                       float eps_high, float beta, hipStream_t s);
hipError_t launch_prepare(const int32_t* host_words, int n_words, int* dev_tab, uint32_t* tag_block, const ReserveTag& tag,
                          int tag_mode, bool with_schedule, int n_groups, int64_t total_tokens, int n256, int n128,
                          const Schedule& sched, hipStream_t s);

// Packings whose 256-row workgroups would run fewer 64-key steps than this on average take the kernels'
// 128-row shape (two workgroups per CU).  SP_ATTN_SMALL_STEPS overrides the default, for measurements.
int small_shape_steps();

// Number of 64-key steps that the workgroups of this packing run with row tiles of `bm` rows (per q head; host
// arithmetic on the segment table), and the number of such workgroups.
inline void key_steps(const Problem& p, int bm, int64_t& steps, int64_t& tiles) {
    const int32_t* tab = p.host_table;
    steps = 0; tiles = 0;
    for (int g = 0; g < p.n_groups; ++g) {
        const int32_t* e = tab + TAB_HEADER + TAB_GROUP_WORDS * g;
        const int Lp = e[1], Tg = e[2], G = e[4];
        const int32_t* roff = tab + e[3];
        for (int t0 = 0; t0 < Tg; t0 += bm, ++tiles) {
            const int t1 = t0 + bm < Tg ? t0 + bm : Tg;
            const int n1 = ((Lp < t1 ? Lp : t1) + 63) / 64;
            steps += n1;
            if (t1 > Lp) {
                const int first = t0 > Lp ? t0 : Lp;          // first response row: its segment start opens the range
                int lo = 0, hi = G;
                while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (roff[mid] <= first) lo = mid; else hi = mid; }
                const int k2b = roff[lo] / 64 > n1 ? roff[lo] / 64 : n1;
                steps += (t1 + 63) / 64 - k2b;
            }
        }
    }
}

// Which workgroup shape the forward and the dq pass take.  The 128-row shape executes less work that no row
// of a tile needs (fewer rows ride along through the key tiles of other responses and past their own
// diagonal) and overlaps the fixed costs of two workgroups per CU, but pays for it: twice the tile copies per
// MFMA and a barrier per step.  Measured on packings from 3 K to 270 K tokens the price is about 3 % of
// the loop, so the small shape is taken when it saves more executed steps than that.  The knob, when set,
// replaces the rule by a threshold on the mean number of steps of a 256-row workgroup.
inline bool use_small_shape(const Problem& p) {
    int64_t s256, t256, s128, t128;
    key_steps(p, 256, s256, t256);
    const int knob = small_shape_steps();
    if (knob >= 0) return t256 > 0 && (double)s256 / (double)t256 < (double)knob;
    key_steps(p, 128, s128, t128);
    return 0.5 * (double)s128 * 1.03 < (double)s256;
}


// Packings that the bandwidth-shaped bf16 rowsum kernel takes (its per-head sums of 16 tokens fit its LDS)
inline bool rowsum_fast_path(const Problem& p) { return p.head_dim == 128 && (size_t)p.Hq * 16 * sizeof(float) <= 32768; }

inline int count_tiles(const Problem& p, int bm) {
    int n = 0;
    for (int g = 0; g < p.n_groups; ++g) n += (p.host_group_tokens[g] + bm - 1) / bm;
    return n;
}

// Small problems leave most CUs idle in the dkdv pass (one workgroup per 128 keys and kv head):
// below this many workgroups the pass is split over the q heads of each kv head, through fp32
// partial sums in the workspace.  Both the workspace size and the launch use this rule.
inline bool dkdv_head_split(int64_t total_tokens, int n_groups, int Hq, int Hkv) {
    return Hq > Hkv && (total_tokens / 128 + n_groups) * Hkv <= 192;
}

}  // namespace sp
