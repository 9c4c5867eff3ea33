/*
 * sp_attn.h -- C ABI of the shared-prompt attention library for AMD MI355X (gfx950).
 *
 * The operation is the attention of Section 4.3 ("Shared-Prompt Attention") of
 * "Periodic Asynchrony: An On-Policy Approach for Accelerating LLM Reinforcement
 * Learning": one group's tokens are packed as [prompt | resp_1 | ... | resp_G]
 * (modification 1 of that section), and the mask (modification 3) lets a prompt
 * token attend causally to the prompt, and a token of response i attend to the
 * whole prompt and causally to response i, never to another response.  The result
 * equals G ordinary causal attentions over [prompt | resp_i] (closing paragraph of
 * the section), with the prompt's key/value gradients summed over the G responses.
 *
 * Conventions common to every entry point
 *   - Tensors are DEVICE pointers, row-major and contiguous, token-major:
 *       q, o, d_o, dq : [T_total, n_q_heads,  head_dim]
 *       k, v, dk, dv  : [T_total, n_kv_heads, head_dim]
 *       lse           : [n_q_heads, T_total]  float32, natural log of
 *                       sum over allowed keys of exp(softmax_scale * <q, k>)
 *     Element type is bf16 (SP_BF16) or float32 (SP_F32, a plain-ALU debug path).
 *     Base pointers must be 16-byte aligned.
 *   - q head h reads kv head h / (n_q_heads / n_kv_heads) (contiguous blocks).
 *   - q and k arrive already position-encoded: the restarted position ids of
 *     modification 2 are applied by the caller before this call.
 *   - Lengths (prompt_len, resp_lens[...]) are HOST integers and are consumed
 *     before the call returns.  Zero-length responses and prompt_len == 0 are
 *     legal; a group must hold at least one token.
 *   - The caller owns all device memory including the workspace.  The library
 *     never allocates, frees or synchronises; work is enqueued on `stream`
 *     (a hipStream_t passed as void*, NULL = the default stream) and the call
 *     returns at once.  Outputs are overwritten, inputs are never modified.
 *     A workspace carries nothing from call to call except the optional forward-to-backward
 *     reserve described at sp_attn_reserve_bytes().
 *   - Every call returns sp_status and sp_attn_last_error() describes a failure.  Arguments,
 *     geometry and workspace are checked before anything is enqueued: on SP_ERR_INVALID_ARG,
 *     SP_ERR_UNSUPPORTED and SP_ERR_WORKSPACE no work has been enqueued and no memory is touched.
 *     SP_ERR_DEVICE means the HIP runtime rejected one of the call's launches; launches of the
 *     same call that preceded it (the segment-table upload into the workspace, earlier stages)
 *     stay enqueued, so the workspace and the outputs are then undefined.
 */
#ifndef SP_ATTN_H
#define SP_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SP_OK = 0,
    SP_ERR_INVALID_ARG = 1,   /* null/misaligned pointer, negative length, empty group,
                                 n_q_heads % n_kv_heads != 0, scale not finite or <= 0 */
    SP_ERR_UNSUPPORTED = 2,   /* head_dim or dtype the kernels do not implement */
    SP_ERR_WORKSPACE = 3,     /* workspace NULL or smaller than sp_attn_workspace_bytes() */
    SP_ERR_DEVICE = 4         /* the HIP runtime reported a launch error */
} sp_status;

typedef enum {
    SP_BF16 = 0,              /* bf16 tensors, bf16 MFMA contractions, fp32 softmax/accumulate;
                                 head_dim must be 128 */
    SP_F32 = 1                /* float32 tensors, plain-ALU debug path; head_dim 64 or 128 */
} sp_dtype;

/* Which kernel schedule the forward uses.  SP_SCHED_SHARED is the product path:
 * wholly masked tiles are skipped and prompt key/value tiles are shared by the
 * query tiles of all responses.  SP_SCHED_NAIVE_CAUSAL is a measurement baseline
 * that visits every tile at or below the diagonal of the packed sequence and
 * applies the mask element by element; its results are identical. */
typedef enum { SP_SCHED_SHARED = 0, SP_SCHED_NAIVE_CAUSAL = 1 } sp_schedule;

/* Bytes of device workspace a call needs (Section 4.3 has no counterpart: this is
 * where the segment table and, for the backward, D = rowsum(dO * O) live).
 * total_tokens = sum over groups of prompt_len + sum(resp_lens); total_responses =
 * sum of G over groups.  Returns 0 for arguments no call would accept. */
size_t sp_attn_workspace_bytes(int is_bwd, int64_t total_tokens, int32_t n_groups,
                               int64_t total_responses, int32_t n_q_heads,
                               int32_t n_kv_heads, int32_t head_dim, sp_dtype dtype);

/* Forward-to-backward reserve (bf16 only; 0 for SP_F32).  The backward starts from
 * D = rowsum(d_o * o), and o reaches it rounded to bf16; where one key dominates a row, that
 * rounding is the largest error of dq and dk.  A forward whose workspace has at least
 *     sp_attn_workspace_bytes(1, ...) + sp_attn_reserve_bytes(...)
 * bytes also leaves there what the rounding of o dropped (o_fp32 - o, itself in bf16; o is
 * unchanged), and a backward that is handed THE SAME workspace, not used by any other call in
 * between, forms D from o plus that residual.  Nothing else changes hands: same arguments, same
 * outputs.  The reserve is protected by a tag at the head of the workspace, naming the o / lse
 * pointers and the shape it belongs to; every call of this library rewrites or re-validates the tag
 * on the device before it writes to a workspace, so a backward that is given a smaller, another,
 * or a since-reused workspace finds no valid reserve and computes D from the bf16 o alone (the
 * result is then what it is without the reserve, never worse).  The explicit o_lo tensor of the
 * _ex entry points does the same through caller memory and takes precedence.  Not written by
 * sp_attn_fwd_multi or by the naive baseline schedule. */
size_t sp_attn_reserve_bytes(int64_t total_tokens, int32_t n_q_heads, int32_t head_dim, sp_dtype dtype);

/* Forward for one group (Section 4.3, modifications 1 and 3): writes
 * o [T, n_q_heads, head_dim] and lse [n_q_heads, T], T = prompt_len + sum(resp_lens).
 * resp_lens: HOST array of G >= 0 entries (may be NULL when G == 0). */
sp_status sp_attn_fwd(const void* q, const void* k, const void* v,
                      void* o, float* lse,
                      int32_t prompt_len, const int32_t* resp_lens, int32_t G,
                      int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                      float softmax_scale, sp_dtype dtype,
                      void* workspace, size_t workspace_bytes, void* stream);

/* Backward for one group: given o and lse from sp_attn_fwd and the upstream
 * gradient d_o (all T rows, prompt rows included), overwrites dq, dk, dv with the
 * exact gradient of sum(o * d_o).  The prompt rows of dk/dv accumulate the
 * contributions of the later prompt rows and of every row of all G responses
 * (the equivalence grad L_shared = sum_k grad L_k of Section 4.3); each kv head
 * sums over the q heads that read it.  Deterministic: no atomics are used. */
sp_status sp_attn_bwd(const void* q, const void* k, const void* v,
                      const void* o, const float* lse, const void* d_o,
                      void* dq, void* dk, void* dv,
                      int32_t prompt_len, const int32_t* resp_lens, int32_t G,
                      int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                      float softmax_scale, sp_dtype dtype,
                      void* workspace, size_t workspace_bytes, void* stream);

/* Batched forms: n_groups independent groups packed back to back along the token
 * axis (samples at their native lengths, no padding, as in Section 5).  Group g has
 * prompt_lens[g] prompt tokens and Gs[g] responses whose lengths are the next Gs[g]
 * entries of resp_lens_flat.  All three arrays are HOST memory.  Several weight
 * sets (policy / old policy / reference, Section 4.2.1) are simply more groups.
 * `schedule` selects SP_SCHED_SHARED or the naive baseline (forward only). */
sp_status sp_attn_fwd_batched(const void* q, const void* k, const void* v,
                              void* o, float* lse,
                              int32_t n_groups, const int32_t* prompt_lens,
                              const int32_t* Gs, const int32_t* resp_lens_flat,
                              int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                              float softmax_scale, sp_dtype dtype, sp_schedule schedule,
                              void* workspace, size_t workspace_bytes, void* stream);

sp_status sp_attn_bwd_batched(const void* q, const void* k, const void* v,
                              const void* o, const float* lse, const void* d_o,
                              void* dq, void* dk, void* dv,
                              int32_t n_groups, const int32_t* prompt_lens,
                              const int32_t* Gs, const int32_t* resp_lens_flat,
                              int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                              float softmax_scale, sp_dtype dtype,
                              void* workspace, size_t workspace_bytes, void* stream);

/* The backward runs in three stages that a caller may enqueue separately, e.g. to time them:
 *   SP_BWD_STAGE_ROWSUM  D[h, t] = sum_j d_o[t,h,j] * o[t,h,j] (o plus the forward's rounding residual
 *                        when the workspace holds a valid reserve or o_lo is given) and
 *                        lse * log2(e) -> workspace.  Needs o, d_o, lse; on the bf16 path also q, k, v:
 *                        rows that see at most 64 keys get D from its definition sum_s P*dP in fp32.
 *   SP_BWD_STAGE_DQ      dq      (needs D in the same workspace; o unused).  On the bf16 path it
 *                        also REPLACES D in the workspace by sum_s P*dP, the same quantity
 *                        evaluated in fp32 without the bf16 rounding of o, and writes the dq of rows
 *                        that see at most 64 keys in a separate small kernel (fp32 dS).
 *   SP_BWD_STAGE_DKDV    dk, dv  (needs D in the same workspace; o unused)
 * Ordering on one workspace: ROWSUM first; then DQ and DKDV one after the other, never concurrently
 * (DQ rewrites the D plane that DKDV reads: overlapping them, e.g. on two streams, is a data race).
 * Either order of the two is correct; DKDV after DQ, which is what sp_attn_bwd* do, is the more
 * accurate one when no reserve is used, and the only one whose results are bitwise repeatable from
 * run to run.  To overlap the two gradient passes, give each its own workspace and run ROWSUM on
 * both.  Output pointers of stages that are not requested may be NULL.
 * A bf16 call that holds both ROWSUM and DQ (and is not in response-rows mode) runs no separate
 * rowsum kernel: the dq pass, which loads every row of d_o anyway, forms D and lse * log2(e) in its
 * prologue, with the same operations in the same order, so that the results equal those of the
 * stages enqueued one by one bit for bit.
 * sp_attn_bwd_batched(...) is this call with SP_BWD_STAGE_ALL. */
#define SP_BWD_STAGE_ROWSUM 1u
#define SP_BWD_STAGE_DKDV   2u
#define SP_BWD_STAGE_DQ     4u
#define SP_BWD_STAGE_ALL    7u
sp_status sp_attn_bwd_batched_stages(const void* q, const void* k, const void* v,
                                     const void* o, const float* lse, const void* d_o,
                                     void* dq, void* dk, void* dv,
                                     int32_t n_groups, const int32_t* prompt_lens,
                                     const int32_t* Gs, const int32_t* resp_lens_flat,
                                     int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                     float softmax_scale, sp_dtype dtype, uint32_t stages,
                                     void* workspace, size_t workspace_bytes, void* stream);

/* sp_attn_bwd_batched for callers that cannot allocate or hand over device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results
 * (bitwise) as sp_attn_bwd_batched, without the workspace: the segment table, D and the other
 * intermediates live in an array of SP_STATIC_SCRATCH_BYTES bytes that is part of the library's
 * device image (every GPU the library is used on holds its own copy until the process ends).  The
 * call allocates and frees nothing, on the host's HIP side or through any library.
 *   - A problem whose sp_attn_workspace_bytes(1, ...) exceeds SP_STATIC_SCRATCH_BYTES is rejected with
 *     SP_ERR_WORKSPACE before anything is enqueued (bf16: about n_q_heads * T_total <= 4e6).
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 *     streams, or host threads) race on it.  Calls ordered on one stream are safe; every call
 *     rewrites all it reads, so nothing carries over from one call to the next.
 *   - Runs on the device that is current at the call; SP_ERR_DEVICE if its address of the array
 *     cannot be obtained. */
#define SP_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
sp_status sp_attn_bwd_batched_static(const void* q, const void* k, const void* v,
                                     const void* o, const float* lse, const void* d_o,
                                     void* dq, void* dk, void* dv,
                                     int32_t n_groups, const int32_t* prompt_lens,
                                     const int32_t* Gs, const int32_t* resp_lens_flat,
                                     int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                     float softmax_scale, sp_dtype dtype, void* stream);

/* Micro-batches that share a prompt.  When the G responses of a prompt are spread over several
 * micro-batches (the paper's runs share 16 of 32 rollouts per micro-batch), each micro-batch packs
 * [prompt | its responses] and the gradient of the group is the sum over its members (Section 3,
 * Eq. 1).  The prompt rows are then the same in every micro-batch, and two flags let a caller
 * compute them once instead of once per micro-batch:
 *   SP_FLAG_RESPONSE_ROWS     forward: o and lse are written for response rows only (prompt rows
 *                             of the outputs keep their contents, e.g. those of the micro-batch
 *                             that ran in full).  backward: dq is written for response rows only
 *                             and only response rows contribute to dk, dv -- exactly the backward
 *                             for an upstream gradient that is zero on the prompt rows, without
 *                             visiting the prompt-by-prompt part of the mask.
 *   SP_FLAG_ACCUMULATE_DKDV   backward: dk, dv are ADDED to what the buffers hold (read-modify-write
 *                             in the output dtype) instead of overwritten, so the prompt's dk/dv
 *                             can be summed over micro-batches in place (each accumulation
 *                             rounds the running sum to the output dtype once more).
 *                             With SP_FLAG_RESPONSE_ROWS the backward uses o and lse on response
 *                             rows only; their prompt rows may hold anything (the buffers are
 *                             still full-size: prompt rows may be read and discarded).
 * The prompt rows' own backward (plain causal attention over the prompt, with the upstream
 * gradient of the prompt rows summed over the micro-batches) is an ordinary call with G = 0.
 * The _ex entry points are sp_attn_fwd_batched / sp_attn_bwd_batched_stages with a flags word and
 * one optional tensor; flags = 0 and o_lo = NULL give those calls.  SP_ERR_INVALID_ARG for unknown
 * bits, or ACCUMULATE on a forward.
 *   o_lo   DEVICE [T_total, n_q_heads, head_dim] bf16, or NULL.  The backward starts from
 *          D = rowsum(d_o * o), and o is stored rounded to bf16; in rows dominated by one key that
 *          rounding is the largest error of dq.  When the forward is given o_lo it also stores
 *          what the rounding dropped (o_fp32 - o, itself rounded to bf16); handing the same buffer
 *          to the backward makes D use o + o_lo.  bf16 only (SP_ERR_UNSUPPORTED with SP_F32). */
#define SP_FLAG_RESPONSE_ROWS   1u
#define SP_FLAG_ACCUMULATE_DKDV 2u
sp_status sp_attn_fwd_batched_ex(const void* q, const void* k, const void* v, void* o, float* lse,
                                 int32_t n_groups, const int32_t* prompt_lens,
                                 const int32_t* Gs, const int32_t* resp_lens_flat,
                                 int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                 float softmax_scale, sp_dtype dtype, sp_schedule schedule,
                                 uint32_t flags, void* o_lo,
                                 void* workspace, size_t workspace_bytes, void* stream);
sp_status sp_attn_bwd_batched_ex(const void* q, const void* k, const void* v,
                                 const void* o, const float* lse, const void* d_o,
                                 void* dq, void* dk, void* dv,
                                 int32_t n_groups, const int32_t* prompt_lens,
                                 const int32_t* Gs, const int32_t* resp_lens_flat,
                                 int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                 float softmax_scale, sp_dtype dtype, uint32_t stages,
                                 uint32_t flags, const void* o_lo,
                                 void* workspace, size_t workspace_bytes, void* stream);

/* Forward for several tensor sets that share ONE packing, in one launch: the policy, old-policy
 * and reference models of a GRPO step score the same packed sequences, so their three
 * attention forwards differ only in q, k, v (Section 3.2: all log-probabilities of a
 * micro-step are evaluated together; Section 4.3 packing).  The segment table is built and
 * uploaded once, the mask classification and the block schedule are shared, and set i's blocks
 * read q[i], k[i], v[i] and write o[i], lse[i].  Results are bitwise those of n_sets separate
 * sp_attn_fwd_batched calls.
 *   n_sets        1 .. SP_MAX_SETS
 *   q, k, v, o, lse   HOST arrays of n_sets DEVICE pointers (layouts as in sp_attn_fwd);
 *                 the arrays are read before the call returns
 *   the rest      as sp_attn_fwd_batched (schedule: shared-prompt).  The workspace is that of
 *                 one forward: sp_attn_workspace_bytes(0, ...).
 * Errors as sp_attn_fwd; SP_ERR_INVALID_ARG also for n_sets out of range or a NULL array. */
#define SP_MAX_SETS 4
sp_status sp_attn_fwd_multi(int32_t n_sets, const void* const* q, const void* const* k,
                            const void* const* v, void* const* o, float* const* lse,
                            int32_t n_groups, const int32_t* prompt_lens,
                            const int32_t* Gs, const int32_t* resp_lens_flat,
                            int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                            float softmax_scale, sp_dtype dtype,
                            void* workspace, size_t workspace_bytes, void* stream);

/* Rotary position embedding with the shared-prompt position indices (Section 4.3,
 * modification 2): the prompt keeps positions 0 .. prompt_len-1 and EVERY response starts again
 * at prompt_len, so attention over the pack equals per-sample training including positions.
 * Half-split rotary form (the Qwen-family convention): theta_i = rope_base^(-2i/head_dim),
 * pair (x[i], x[i + head_dim/2]) of a token at position p turns by the angle p * theta_i
 * (theta_i and the product are formed in double precision and reduced to [-pi, pi] before the
 * fp32 sine and cosine).
 *   x, y          DEVICE [T_total, n_heads, head_dim], dtype elements; y may equal x (in place).
 *                 Call it on q (n_q_heads) and on k (n_kv_heads) before sp_attn_fwd; v is not rotated.
 *   inverse       0: rotate by +angle.  1: rotate by -angle, which turns the gradients that
 *                 sp_attn_bwd returns for the rotated q / k into gradients for the unrotated ones.
 *   packing       as sp_attn_fwd_batched.  head_dim 64 or 128 for either dtype.
 *   workspace     DEVICE, at least sp_attn_workspace_bytes(0, T_total, n_groups, total_responses,
 *                 n_heads, n_heads, head_dim, dtype) bytes (it holds the segment table).
 * Asynchronous on `stream`; errors as sp_attn_fwd (SP_ERR_INVALID_ARG also for rope_base <= 1). */
sp_status sp_attn_rope(const void* x, void* y, int32_t n_heads, int32_t inverse,
                       int32_t n_groups, const int32_t* prompt_lens,
                       const int32_t* Gs, const int32_t* resp_lens_flat,
                       int32_t head_dim, double rope_base, sp_dtype dtype,
                       void* workspace, size_t workspace_bytes, void* stream);

/* The same rotation applied to q (n_q_heads) and to k (n_kv_heads) in ONE launch: one segment-table
 * upload, one position lookup per token and one set of angles serve both tensors (with inverse = 1:
 * dq and dk).  Results are bitwise those of two sp_attn_rope calls.  Arguments as sp_attn_rope; the
 * workspace is that of the q call. */
sp_status sp_attn_rope_qk(const void* q, void* q_out, int32_t n_q_heads,
                          const void* k, void* k_out, int32_t n_kv_heads, int32_t inverse,
                          int32_t n_groups, const int32_t* prompt_lens,
                          const int32_t* Gs, const int32_t* resp_lens_flat,
                          int32_t head_dim, double rope_base, sp_dtype dtype,
                          void* workspace, size_t workspace_bytes, void* stream);

/* ---- Response-token loss (Section 4.3, modification 4; Section 2 objective) ------------------
 * The loss of the pack is a cross-entropy over its RESPONSE tokens; prompt rows are discarded.
 * All three calls take the packing of sp_attn_fwd_batched and touch response rows only: prompt
 * rows of every per-token tensor are neither read nor written.  Workspace (DEVICE): at least
 * sp_attn_loss_workspace_bytes(T_total, n_groups, total_responses) bytes.  Asynchronous on
 * `stream`; errors as sp_attn_fwd.
 *
 * sp_attn_logprob_fwd   logp[t] = logits[t, labels[t]] - log sum_v exp(logits[t, v]); also returns
 *                       that log-sum-exp in lse[t] for the backward.  A label outside [0, vocab)
 *                       gives logp = -inf without touching memory.
 *     logits  DEVICE [T_total, vocab], dtype elements, row-major;  labels  DEVICE int32 [T_total]
 *     (the target of each row; the next-token shift is the caller's);  logp, lse  DEVICE fp32 [T_total]
 * sp_attn_logprob_bwd   dlogits[t, v] = g[t] * (1[v == labels[t]] - exp(logits[t, v] - lse[t]))
 *     g  DEVICE fp32 [T_total] = dL/dlogp;  dlogits  DEVICE [T_total, vocab], dtype elements
 *     (may not alias logits)
 * sp_attn_grpo_loss     loss = -1/R sum_k (L_k - beta D_k) over the R non-empty responses, with one
 *                       advantage A_k per response (adv: DEVICE fp32 [total_responses], responses in
 *                       packing order over all groups), |o_k| its token count and, per token,
 *                         r = exp(logp - logp_old),  L_k = 1/|o_k| sum min(r A_k, clip(r, 1-eps_low, 1+eps_high) A_k),
 *                         u = logp_ref - logp,       D_k = 1/|o_k| sum (exp(u) - u - 1).
 *                       The paper names these terms without printing them; this is the GRPO form.
 *     logp, logp_old, logp_ref  DEVICE fp32 [T_total];  loss  DEVICE fp32 [1];
 *     g  DEVICE fp32 [T_total] = dloss/dlogp (feeds sp_attn_logprob_bwd).  Bitwise repeatable. */
size_t    sp_attn_loss_workspace_bytes(int64_t total_tokens, int32_t n_groups, int64_t total_responses);
sp_status sp_attn_logprob_fwd(const void* logits, const int32_t* labels, float* logp, float* lse,
                              int64_t vocab, int32_t n_groups, const int32_t* prompt_lens,
                              const int32_t* Gs, const int32_t* resp_lens_flat, sp_dtype dtype,
                              void* workspace, size_t workspace_bytes, void* stream);
sp_status sp_attn_logprob_bwd(const void* logits, const int32_t* labels, const float* lse,
                              const float* g, void* dlogits, int64_t vocab,
                              int32_t n_groups, const int32_t* prompt_lens,
                              const int32_t* Gs, const int32_t* resp_lens_flat, sp_dtype dtype,
                              void* workspace, size_t workspace_bytes, void* stream);
sp_status sp_attn_grpo_loss(const float* logp, const float* logp_old, const float* logp_ref,
                            const float* adv, float eps_low, float eps_high, float beta,
                            float* loss, float* g,
                            int32_t n_groups, const int32_t* prompt_lens,
                            const int32_t* Gs, const int32_t* resp_lens_flat,
                            void* workspace, size_t workspace_bytes, void* stream);

/* The segment table that every call builds from its host arrays and hands to its kernels (Section
 * 4.3, packing and mask: the table is the only form in which they reach the device).  Written to
 * HOST memory `words` (capacity in int32 words); *n_words receives the count needed, also when
 * the capacity is too small (then SP_ERR_WORKSPACE and nothing is written) or words is NULL.
 * Layout, all int32:
 *   [0] n_groups  [1] total tokens  [2] table words  [3] 0
 *   group g at 4 + 8 g: { first packed token, prompt_len, tokens T_g, index of its offsets, G,
 *                         256-row tiles in earlier groups, 128-key tiles in earlier groups, 0 }
 *   then per group G + 1 group-local offsets: prompt_len, ends of responses 1 .. G (the last = T_g).
 * No device work; for tools and tests.  Errors as the host checks of sp_attn_fwd_batched. */
sp_status sp_attn_segment_table(int32_t n_groups, const int32_t* prompt_lens, const int32_t* Gs,
                                const int32_t* resp_lens_flat, int32_t* words, size_t capacity,
                                size_t* n_words);

/* Measurement aid (no counterpart in the paper): a loop of nothing but bf16 32x32x16 MFMAs, so that
 * the attention kernels' rates can be read against what the matrix cores of this chip sustain.
 *   lds_operands  0: both operands in registers; 1: one operand read from LDS per MFMA (as in the
 *                 forward and the dq pass); 2: both read from LDS
 *   a, b          DEVICE, 16-byte aligned, 8 * 512 * 8 bf16 each: the operand values (random values
 *                 draw the power real data draws; constants do not)
 *   iters         iterations of 16 MFMAs per wave;  n_blocks  workgroups of 8 waves (256 = one per CU)
 *   out           DEVICE float[512], overwritten
 * Executes n_blocks * 8 * iters * 16 * 32768 FLOPs.  Asynchronous on `stream`.
 * SP_ERR_INVALID_ARG for a NULL/misaligned pointer or a count < 1. */
sp_status sp_attn_mfma_ceiling(int32_t lds_operands, const void* a, const void* b, int32_t iters,
                               int32_t n_blocks, float* out, void* stream);

/* Measurement aid (no counterpart in the paper): the rate at which this chip adds 64 x 128 fp32 tiles
 * into a [rows, heads, 128] fp32 accumulator with memory atomics -- what a backward that produced dQ, dK
 * and dV in one pass would have to do for every (key tile, row tile, q head), 4 bytes per allowed pair
 * and q head.  The two-pass backward of this library exists because of the figure this returns.
 *   buf      DEVICE float[rows * heads * 128], rows a multiple of 64; its contents are added to
 *   steps    tiles added per workgroup;  n_blocks  workgroups of 512 threads
 *   layout   0: half-waves cover 128 contiguous bytes of a row; 1: lanes scatter as an MFMA accumulator
 * Adds n_blocks * steps * 32768 bytes.  Asynchronous on `stream`; SP_ERR_INVALID_ARG for bad counts. */
sp_status sp_attn_probe_atomic_add(float* buf, int64_t rows, int32_t heads, int32_t steps, int32_t n_blocks,
                                   int32_t layout, void* stream);

/* Which workgroup shape a bf16 call on this packing takes for the forward and the dq pass: *rows = 256
 * or 128 (see sp_attn_set_small_shape_steps below for the rule).  Optionally also the number of 64-key
 * steps that the workgroups of either tiling run per q head (the quantities the rule compares; the
 * count for 128-row tiles is in steps of half the rows).  Host arithmetic on the lengths (Section 4.3:
 * the key ranges of the three terms of its complexity split); no device work; for tools and tests.
 * Errors as the host checks of sp_attn_fwd_batched. */
sp_status sp_attn_row_tile(int32_t n_groups, const int32_t* prompt_lens, const int32_t* Gs,
                           const int32_t* resp_lens_flat, int32_t* rows, int64_t* steps_256, int64_t* steps_128);

/* Tuning knob, process-wide (no counterpart in the paper).  The bf16 kernels come in two workgroup
 * shapes: 256 query rows with one workgroup per CU, for long key loops, and 128 rows with two
 * workgroups per CU, whose fixed per-workgroup costs overlap and which execute less work that no row of
 * a tile needs, for batches of short or ragged groups.  By default a call (forward, dq pass) takes the
 * small shape when that saves more than 3 % of the executed 64-key steps (host arithmetic on the
 * lengths).  With the knob set, it takes the small shape when a 256-row workgroup of its packing would run
 * fewer than `steps` such steps on average: 0 = always the large shape; a large value = always the small
 * one; negative = back to the default rule.  Results do not depend on the shape beyond rounding order.
 * For measurements and tests; safe to call at any time between calls. */
void sp_attn_set_small_shape_steps(int32_t steps);

/* Text of the most recent error on the calling thread ("" if none).  The pointer
 * refers to thread-local static storage; the caller must not free it. */
const char* sp_attn_last_error(void);

/* Library version, "major.minor". */
const char* sp_attn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SP_ATTN_H */
