/*
 * dlm.h -- C ABI of libdlm: one denoising step of a masked / block diffusion
 * language model rollout on one AMD MI355X (gfx950).
 *
 * The step (reverse process of a masked diffusion LM; paper Section 2.1, Eq. 1-3,
 * and the rollout paragraph of Section 3.4):
 *   1. dlm_block_attn         the block being denoised attends to the cached
 *                             context and to itself;
 *   2. dlm_lmhead_confidence  the mask predictor's categorical (Eq. 2) is reduced,
 *                             per masked position, to its arg-max token and that
 *                             token's probability, without storing logits;
 *   3. dlm_unmask_commit      a threshold or fixed-count rule (Section 4.1 schedule)
 *                             fixes several positions at once and writes the
 *                             block's K/V back into the cache;
 *   dlm_kv_refresh            block-boundary cache refresh (strided 16-bit copy).
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless its name starts with host_.  The
 *     argument structs themselves live in host memory.
 *   - bf16 tensors are passed as const void*; strides are in ELEMENTS; the
 *     innermost (head_dim / hidden) axis is contiguous.
 *   - The caller owns every buffer, including workspaces; the library allocates
 *     no device memory and keeps no pointer after a call's work has completed.
 *   - Calls validate on the host, enqueue on the HIP stream passed as `stream`
 *     (a hipStream_t; NULL = the default stream) and return without
 *     synchronising.  Outputs are valid once the stream has been synchronised.
 *   - Return value: DLM_OK or a negative DLM_ERR_* code; nothing aborts or
 *     throws.  dlm_last_error() gives a thread-local description of the last
 *     failure on the calling thread.
 *   - struct_size must be set to sizeof(the struct) by the caller.
 */
#ifndef DLM_H
#define DLM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DLM_OK                 0
#define DLM_ERR_INVALID_ARG   (-1)  /* null / negative / inconsistent argument                */
#define DLM_ERR_UNSUPPORTED   (-2)  /* valid but not implemented (e.g. head_dim not 64 / 128) */
#define DLM_ERR_WORKSPACE     (-3)  /* workspace missing or smaller than *_workspace_bytes    */
#define DLM_ERR_HIP           (-4)  /* a HIP runtime call failed (launch error)               */

#define DLM_MASK_FULL          0    /* every query sees every key (masked diffusion LM)       */
#define DLM_MASK_BLOCK_CAUSAL  1    /* key visible iff its block index <= the query's (Eq. 3) */

#define DLM_CONF_TOKEN_PROB    0    /* confidence = probability of the chosen token                          */
#define DLM_CONF_MARGIN        1    /* confidence = p(top-1) - p(top-2)                                      */
#define DLM_CONF_NEG_ENTROPY   2    /* confidence = sum_v p_v log p_v (0 = one-hot, -log V = uniform)         */

#define DLM_RULE_THRESHOLD     0
#define DLM_RULE_TOPK          1

#define DLM_WB_NONE            0
#define DLM_WB_BLOCK_WHEN_DONE 1    /* copy the whole block's K/V when a sequence's last masked position commits */
#define DLM_WB_COMMITTED_ROWS  2    /* copy the K/V rows of the positions committed by this call */
#define DLM_WB_WHILE_ACTIVE    3    /* copy the whole block's K/V for every sequence that entered this call with masked positions */

/* Which blocks of a segment a query may see under DLM_MASK_BLOCK_CAUSAL (kb, qb = block index of key, query) */
#define DLM_SEG_CAUSAL         0    /* kb <= qb: the query's block and every earlier one                */
#define DLM_SEG_EARLIER_BLOCKS 1    /* kb <  qb: e.g. the clean copy x_0 seen from a noisy block (Eq. 3) */
#define DLM_SEG_SAME_BLOCK     2    /* kb == qb: e.g. the noisy copy x_t seen from its own block (Eq. 3) */

/* One segment of keys/values: k, v are bf16 [B, Hkv, len, d] addressed as
 * base + b*stride_b + h*stride_h + t*stride_t + c.  len == 0 means "absent".
 * pos0 is the absolute sequence position of row 0 (block-causal mask only).
 * rule: one of DLM_SEG_* (block-causal mask only; must be 0 under DLM_MASK_FULL). */
typedef struct dlm_kv_seg {
    const void *k, *v;
    int32_t len;
    int32_t pos0;
    int64_t stride_b, stride_h, stride_t;
    int32_t rule;
} dlm_kv_seg;

/* ------------------------------------------------------------------------- *
 * dlm_block_attn -- O = softmax(scale * Q K^T) V for a block of Lq query rows
 * per sequence against the concatenation [prefix | block | suffix] of KV
 * segments, with grouped-query heads (kv head = q head / (Hq / Hkv)).
 *
 * Defines: Section 3.4 "Rollout-side optimization for MDLMs" (KV-cache reuse:
 * the block attends to cached context plus itself; bidirectional, Eq. 2) and
 * the block partition before Eq. 3 (block-causal visibility).
 *
 *   q       bf16 [B, Lq, Hq, d]   (q_stride_b, q_stride_t, q_stride_h)
 *   out     bf16 [B, Lq, Hq, d]   (o_stride_*), written
 *   lse     optional fp32 [B, Hq, Lq] contiguous: natural-log sum of exp(scale*s)
 *   prefix_len_b  optional int32 [B]: only the first prefix_len_b[b] rows of
 *           `prefix` exist for sequence b (0 <= value <= prefix.len)
 *   mask_mode DLM_MASK_BLOCK_CAUSAL: key at absolute position p is visible to
 *           query row i iff floor(p / block_size) <= floor((q_pos0 + i) / block_size)
 *           for a segment with rule DLM_SEG_CAUSAL; the other two rules replace <= by < and ==.
 *           Block-diffusion training over the pair (noisy x_t, clean x_0) of Eq. 3 is two calls:
 *           noisy queries with prefix = clean K/V (EARLIER_BLOCKS) and block = noisy K/V (SAME_BLOCK),
 *           both at pos0 = 0, and clean queries with block = clean K/V (CAUSAL).
 *   scale   <= 0 selects 1/sqrt(d)
 * Arithmetic: bf16 operands, fp32 scores / softmax / accumulation, probabilities
 * rounded to bf16 for the second product, bf16 output.  A row that sees no key
 * gets out = 0 and lse = -inf.
 * Supported: d in {64, 128}; Hq % Hkv == 0; all base pointers 16-byte aligned and
 * all strides multiples of 8 elements.  Lq, Hq/Hkv and segment lengths are arbitrary.
 * workspace: optional.  dlm_block_attn_workspace_bytes(args) is non-zero for shapes that leave most of the chip idle with
 *           one workgroup per row tile (few sequences x KV heads, long context): given that many bytes (16-byte aligned),
 *           the call lets several workgroups share the keys of a row tile (fp32 partial results in the workspace, merged
 *           in a fixed order by a second launch: deterministic).  Without it, or with a smaller buffer, the call runs
 *           unsplit; results then differ by the rounding of another summation order only.
 *   seq_active  optional device int32 [B]: sequence b is skipped (its rows of out and lse are left as they
 *           are) when seq_active[b] == 0.  For denoising steps in which some sequences of the batch have no
 *           masked position left: nothing reads their attention output (the LM head runs on masked rows
 *           only), so the driver passes the previous step's per-sequence count of masked positions.
 *
 * Packed variable-length mode (cu_seqlens != NULL; Section 3.4, training-side optimization: the
 * padding-free bidirectional attention used for SFT, the actor update and log-prob
 * recomputation): the batch is one token-major buffer without PAD rows.
 *   cu_seqlens    device int32 [B + 1], non-decreasing, cu_seqlens[0] = 0; sequence b owns tokens
 *                 [cu_seqlens[b], cu_seqlens[b+1]) and attends only to itself
 *   total_tokens  cu_seqlens[B]
 *   q, out        bf16 [total_tokens, Hq, d]  (stride_t, stride_h; stride_b ignored)
 *   block.k / v   bf16 [total_tokens, Hkv, d] (stride_t, stride_h; stride_b ignored)
 *   Lq = block.len = an upper bound on the sequence lengths (the longest one); a sequence longer than
 *                 that is truncated to its first Lq tokens (queries and keys alike)
 *   prefix, suffix, prefix_len_b must be absent; lse is fp32 [Hq, total_tokens]
 *   block-causal: positions restart in every sequence (query row i at q_pos0 + i, key j at block.pos0 + j).
 * ------------------------------------------------------------------------- */
typedef struct dlm_attn_args {
    uint32_t struct_size;
    int32_t B, Lq, Hq, Hkv, d;
    const void *q;
    int64_t q_stride_b, q_stride_t, q_stride_h;
    dlm_kv_seg prefix, block, suffix;
    const int32_t *prefix_len_b;
    int32_t mask_mode;
    int32_t block_size, q_pos0;
    float scale;
    void *out;
    int64_t o_stride_b, o_stride_t, o_stride_h;
    float *lse;
    void *workspace;
    size_t workspace_bytes;
    const int32_t *cu_seqlens;
    int32_t total_tokens;
    const int32_t *seq_active;
} dlm_attn_args;

int dlm_block_attn(const dlm_attn_args *args, void *stream);
size_t dlm_block_attn_workspace_bytes(const dlm_attn_args *args);

/* ------------------------------------------------------------------------- *
 * dlm_block_attn_bwd -- gradients of dlm_block_attn for training through the attention of a mask
 * predictor (the NELBO objectives of Eq. 2 and Eq. 3 are minimised by gradient descent; the masks are
 * the forward pass's: full, block-causal with per-segment rules, packed variable-length).
 * With P = softmax(scale Q K^T + mask), O = P V and the upstream gradient d_out:
 *   d_v = P^T d_out;   dP = d_out V^T;   dS = P * (dP - rowsum(d_out * O));
 *   d_q = scale dS K;  d_k = scale dS^T Q      (d_k, d_v summed over the query heads of a KV group)
 *
 *   q, out, d_out  bf16 [B, Lq, Hq, d] with their own strides; out and lse are the forward results
 *   lse            fp32, the forward layout ([B, Hq, Lq], or [Hq, total_tokens] in packed mode)
 *   d_q            bf16 [B, Lq, Hq, d] (dq_stride_*), written; NULL: not wanted
 *   d_<seg>_k / _v bf16, laid out exactly like that segment's k / v (same strides), written for every row
 *                  of the segment (zeros where no query sees the key); NULL pair: not wanted.  A tensor that
 *                  serves as K/V in several calls (e.g. the clean copy in block-diffusion training) gets
 *                  one gradient per call; adding them is the caller's.
 *   prefix_len_b is not supported here (ragged caches belong to rollout, not to training).
 * P is recomputed from q, k and lse: no Lq x Lk tensor is stored.  bf16 operands (P and dS are rounded to
 * bf16 for their second products), fp32 accumulation, bf16 results.  No atomics: results are deterministic.
 * workspace: dlm_block_attn_bwd_workspace_bytes(args) bytes, 16-byte aligned (one fp32 per query row and head).
 * Supported sizes and alignment: as dlm_block_attn.
 * ------------------------------------------------------------------------- */
typedef struct dlm_attn_bwd_args {
    uint32_t struct_size;
    int32_t B, Lq, Hq, Hkv, d;
    const void *q;
    int64_t q_stride_b, q_stride_t, q_stride_h;
    const void *out;
    int64_t o_stride_b, o_stride_t, o_stride_h;
    const void *d_out;
    int64_t do_stride_b, do_stride_t, do_stride_h;
    const float *lse;
    dlm_kv_seg prefix, block, suffix;
    int32_t mask_mode;
    int32_t block_size, q_pos0;
    float scale;
    void *d_q;
    int64_t dq_stride_b, dq_stride_t, dq_stride_h;
    void *d_prefix_k, *d_prefix_v, *d_block_k, *d_block_v, *d_suffix_k, *d_suffix_v;
    void *workspace;
    size_t workspace_bytes;
    const int32_t *cu_seqlens;
    int32_t total_tokens;
} dlm_attn_bwd_args;

int dlm_block_attn_bwd(const dlm_attn_bwd_args *args, void *stream);
size_t dlm_block_attn_bwd_workspace_bytes(const dlm_attn_bwd_args *args);

/* ------------------------------------------------------------------------- *
 * dlm_lmhead_confidence -- for each of M selected rows r of `hidden`:
 *   z_v  = (hidden[row(r), :] . w[v, :]) * inv_temperature,  v in [0, V)
 *   z_forbid_token = -inf (when forbid_token >= 0)
 *   tok  = smallest v maximising z_v;  zmax = z_tok;  z2nd = max_{v != tok} z_v
 *   lse  = log sum_v exp(z_v);  conf = exp(zmax - lse)
 *   ztarget = z_{target[r]}  (optional; log p(target) = ztarget - lse, the term
 *             summed by the NELBO of Eq. 2 / Eq. 3)
 * The V logits of a row are never written to memory.
 *
 * Defines: the mask predictor p_theta(x_0 | x_t) of Eq. 2 evaluated at masked
 * positions; "logits-free" fused projection as in Section 3.4.
 *
 *   hidden  bf16 [rows_total, Dh], row stride hidden_stride_row
 *   row_idx optional int32 [M]: row(r) = row_idx[r]; NULL: row(r) = r
 *   m_dev   optional device int32 scalar: the call processes min(M, max(*m_dev,0))
 *           rows (lets the previous step's compaction set the row count without a
 *           host round trip); outputs beyond that count are left untouched
 *   M_expected  0, or the row count the caller expects *m_dev to hold (a guess, not a bound; needs m_dev).
 *           The kernel shape is chosen on the host from M, which a caller that polls the device late only
 *           knows as an upper bound.  When M_expected falls in a smaller shape's range, the call queues that
 *           shape guarded by "*m_dev fits it" and the shape for M guarded by the opposite, so a right
 *           guess runs the better shape and a wrong one costs an empty launch.  Results depend on it only
 *           through the summation order of the shape that ran (rounding).
 *   w       bf16 [V, Dh], row stride w_stride_row
 *   out_scatter  0: outputs are indexed by r; 1: by row(r) (dense per-position arrays)
 *   conf, tok    required; lse, zmax, z2nd, target+ztarget optional.  `target` is
 *           indexed like the outputs.
 * Sampling (sample = 1; stochastic rollouts, e.g. the group of 8 rollouts per prompt of the
 * implementation details in Section 4.1): tok is drawn from softmax(z) by the Gumbel-max identity,
 *   tok = smallest v maximising z_v + g_v,   g_v = -log(-log u_v),   conf = exp(z_tok - lse),
 * while lse, zmax, z2nd and ztarget keep their meaning.  u_v = (2k + 1) / 2^24 with k the top 23 bits of
 * word v % 4 of Philox-4x32-10(counter = (v / 4, row(r), sample_step, sample_stream), key = (low, high
 * 32 bits of sample_seed)): the draw depends on the row's index in `hidden`, not on r or M, and repeats
 * exactly for equal (seed, step, stream).  Callers give every denoising step its own sample_step and
 * every rollout replica its own sample_stream.
 * conf_mode selects what `conf` holds (the score dlm_unmask_commit ranks and thresholds; the paper leaves the
 * confidence of its decoding open, the model families it names decode with the token probability, the top-2
 * margin or the negative entropy): DLM_CONF_TOKEN_PROB (default; the sampled token's probability when sampling),
 * DLM_CONF_MARGIN, DLM_CONF_NEG_ENTROPY; the latter two score the distribution, whichever token is chosen.
 * Arithmetic: bf16 operands, fp32 accumulation and softmax.
 * Supported: Dh % 64 == 0; hidden, w 16-byte aligned; strides multiples of 8.
 * workspace: dlm_lmhead_workspace_bytes(args) bytes (depends on M, V, sample and conf_mode), 16-byte aligned.
 * ------------------------------------------------------------------------- */
typedef struct dlm_lmhead_args {
    uint32_t struct_size;
    int32_t M, Dh, V;
    const void *hidden;
    int64_t hidden_stride_row;
    const int32_t *row_idx;
    const int32_t *m_dev;
    const void *w;
    int64_t w_stride_row;
    float inv_temperature;
    int32_t forbid_token;
    int32_t out_scatter;
    float *conf;
    int32_t *tok;
    float *lse, *zmax, *z2nd;
    const int32_t *target;
    float *ztarget;
    void *workspace;
    size_t workspace_bytes;
    int32_t sample;
    uint32_t sample_step, sample_stream;
    uint64_t sample_seed;
    int32_t conf_mode;
    int32_t M_expected;
} dlm_lmhead_args;

int dlm_lmhead_confidence(const dlm_lmhead_args *args, void *stream);
size_t dlm_lmhead_workspace_bytes(const dlm_lmhead_args *args);

/* dlm_lmhead_confidence_static -- dlm_lmhead_confidence for callers that cannot allocate or pass a
 * workspace: code running under HIP graph capture, tight serving loops that own no allocator, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels, same results; a->workspace / a->workspace_bytes are ignored
 * and the per-tile partials go to a scratch array built into the library (DLM_LMHEAD_STATIC_SCRATCH_BYTES of
 * device memory per GPU the library runs on, held until the process ends).  The call allocates and frees
 * nothing; on its first use on a device it looks up that device's address of the array (no allocation).
 * Limit: dlm_lmhead_workspace_bytes(a) <= DLM_LMHEAD_STATIC_SCRATCH_BYTES (e.g. 1024 rows at V = 152064,
 * 512 rows when sampling), else DLM_ERR_WORKSPACE and nothing is enqueued.
 * All calls on one GPU share the one array: calls that overlap in time on the same GPU (different streams or
 * threads) race; calls on one stream are ordered and safe.  Nothing in the array needs clearing between calls:
 * every partial a call reads was written by that call. */
#define DLM_LMHEAD_STATIC_SCRATCH_BYTES (32u << 20)
int dlm_lmhead_confidence_static(const dlm_lmhead_args *args, void *stream);
size_t dlm_lmhead_static_scratch_bytes(void);

/* ------------------------------------------------------------------------- *
 * dlm_unmask_commit -- per sequence and per commit group of group_len
 * consecutive positions, among positions with mask == 1:
 *   DLM_RULE_THRESHOLD  commit every position with conf >= threshold and, when
 *                       force_top1 != 0, the most confident one (lowest index on ties);
 *   DLM_RULE_TOPK       commit the min(k, #masked) most confident (ties: lowest index).
 * For committed position i: x[b, x_pos0 + i] = tok[b, i]; mask[b, i] = 0.
 * Positions with mask == 0 on entry are neither read for selection nor written.
 *
 * Defines: the reverse-process commit of Section 3.4 (rollout paragraph) with the fixed schedule of Section 4.1 (top-k) or the
 * confidence-threshold parallel decoding the paper adopts for rollout.
 *
 *   conf, tok   dense fp32 / int32 [B, n_pos] contiguous (index b*n_pos + i)
 *   x           int32, row stride x_stride_b, in/out
 *   mask        uint8, row stride mask_stride_b, in/out
 *   commit_now  optional uint8 [B, n_pos]: 1 where this call committed (fully written)
 *   n_commit, remaining   int32 [B]: committed by this call / still masked after it
 *   next_row_idx, next_m  optional: ascending list of flat indices b*n_pos + i that are
 *                         still masked after this call, and its length (device scalar)
 *   commit_step optional int16 [B, n_pos]: `step` is stored where this call committed
 *   writeback   DLM_WB_*: copy rows of src_block (bf16 [B, Hkv, src_block.len, d]) into
 *               cache_k / cache_v (bf16, strides c_stride_*) at rows cache_pos0 + t.
 *               BLOCK_WHEN_DONE: all rows, for sequences whose remaining becomes 0 in this
 *               call with n_commit > 0.  COMMITTED_ROWS: row i for each committed i
 *               (needs src_block.len == n_pos).  WHILE_ACTIVE: all rows, for sequences with
 *               active_in[b] != 0.  Called on every step of a block with active_in = the previous step's
 *               `remaining` (a DIFFERENT buffer from this call's `remaining` and `n_commit`: the copy reads
 *               it while the selection writes those), the cache ends up holding each sequence's
 *               final-step K/V exactly as with BLOCK_WHEN_DONE, but the copy needs nothing this call
 *               computes, so on the single-workgroup path it runs inside the same launch, beside the
 *               selection (one launch fewer per denoising step; block-sized extra writes per step).
 *   active_in   int32 [B], WHILE_ACTIVE only (see above); ignored otherwise
 *   host_remaining_total  optional pointer to ONE int32 in pinned host memory that the device can
 *               address (hipHostMalloc): receives sum_b remaining[b] (>= 0) with a system-scope release
 *               store, so a caller can learn "block finished" without queueing a device-to-host copy:
 *               either it records an event after the call, or it presets the word to a negative value
 *               before the call and watches the word.  Only the single-workgroup path (one commit group per
 *               sequence and B * n_pos <= 16384) supports it; otherwise DLM_ERR_UNSUPPORTED.
 *   host_remaining_max  optional, with host_remaining_total only: ONE more int32 of pinned host memory that
 *               receives max_b remaining[b], stored before the total (a host that has seen the total
 *               sees this value too).  With the forced top-1 of the threshold rule a maximum of 1 (with
 *               the top-k rule a maximum <= k) means that the NEXT step commits everything that is left,
 *               so a host that polls one step late knows a block's last step when it queues it.
 * Selection compares fp32 values; outputs are integers (bit-exact given conf).
 * Limits: 1 <= group_len <= 1024; d % 8 == 0 for write-back.
 * Calls on one stream are ordered; the kernels of one call race with nothing else.
 * ------------------------------------------------------------------------- */
typedef struct dlm_commit_args {
    uint32_t struct_size;
    int32_t B, n_pos, group_len;
    int32_t rule;
    float threshold;
    int32_t force_top1;
    int32_t k;
    const float *conf;
    const int32_t *tok;
    int32_t *x;
    int64_t x_stride_b;
    int32_t x_pos0;
    uint8_t *mask;
    int64_t mask_stride_b;
    uint8_t *commit_now;
    int32_t *n_commit, *remaining;
    int32_t *next_row_idx, *next_m;
    int16_t *commit_step;
    int32_t step;
    int32_t writeback;
    dlm_kv_seg src_block;
    void *cache_k, *cache_v;
    int64_t c_stride_b, c_stride_h, c_stride_t;
    int32_t cache_pos0, Hkv, d;
    int32_t *host_remaining_total;
    const int32_t *active_in;
    int32_t *host_remaining_max;
} dlm_commit_args;

int dlm_unmask_commit(const dlm_commit_args *args, void *stream);

/* dlm_mask_compact -- ascending list of flat indices b*n_pos + i with mask[b, i] != 0
 * into row_idx (capacity B*n_pos) and its length into *m_out (device scalar).
 * Used at block start to seed dlm_lmhead_confidence's row list (masked rows only, Eq. 2). */
int dlm_mask_compact(const uint8_t *mask, int64_t mask_stride_b, int32_t B, int32_t n_pos,
                     int32_t *row_idx, int32_t *m_out, void *stream);

/* dlm_seq_logprob -- per-sequence masked log-likelihood from the LM head's logits-free outputs:
 *   out[b] = weight_b * sum_{i : mask[b, i] != 0} (ztarget[b*n_pos + i] - lse[b*n_pos + i])
 * i.e. the sum of log p_theta(x_0^i | x_t) over the masked positions that the NELBO of Eq. 2 (masked
 * diffusion) and Eq. 3 (per block) weights by 1/t; `weight` (optional fp32 [B], e.g. -1/t) defaults to 1.
 * Serves log-probability recomputation (old-policy / reference policy) without materialising logits:
 * ztarget and lse are the dense (out_scatter = 1) outputs of dlm_lmhead_confidence with `target` set.
 * n_terms (optional int32 [B]) receives the number of masked positions.  fp32 accumulation in a fixed
 * order (deterministic).  mask rows are mask_stride_b apart; ztarget / lse are contiguous [B, n_pos]. */
int dlm_seq_logprob(const float *ztarget, const float *lse, const uint8_t *mask, int64_t mask_stride_b,
                    const float *weight, int32_t B, int32_t n_pos, float *out, int32_t *n_terms, void *stream);

/* dlm_kv_refresh -- copy src K,V [B, Hkv, src->len, d] into the cache at rows
 * [cache_pos0, cache_pos0 + src->len): the block-boundary cache refresh of a
 * KV-cached rollout (Section 3.4).  Bit-exact 16-bit copy; d % 8 == 0, 16-byte
 * aligned bases, strides multiples of 8.  Source and destination must not overlap. */
int dlm_kv_refresh(const dlm_kv_seg *src, int32_t B, int32_t Hkv, int32_t d,
                   void *cache_k, void *cache_v,
                   int64_t c_stride_b, int64_t c_stride_h, int64_t c_stride_t,
                   int32_t cache_pos0, void *stream);

/* dlm_set_option -- process-wide tuning / test knobs (not thread-safe against running calls).  These integers are the
 * ONLY mutable state the library keeps between calls (besides the per-device address of the built-in scratch of
 * dlm_lmhead_confidence_static); every default is the planner's choice, and every setting computes the same function.
 *   "attn_variant"  0 = pick the attention kernel shape from the problem shape (default);
 *                   1 = 32-row workgroups whose wavefronts split the keys (needs g*Lq <= 32, otherwise falls back to 2),
 *                       sized for one workgroup per CU; 12 = the same sized for two (the planner's choice for g*Lq <= 32);
 *                   2 = 128-row; 3 = 256-row workgroups (one per CU);
 *                   4..7 = 128-row workgroups sized for 2, 3, 3, 4 resident workgroups per CU;
 *                   8..10 = key-split alternatives (deeper prefetch, 8 wavefronts) for g*Lq <= 32;
 *                   11 = 32-row key-split workgroups for any row count, the row tiles of one (sequence, KV head) grouped
 *                       on one XCD (chosen when 128-row workgroups would leave most CUs idle and no workspace is given);
 *                   13, 14 = 128-row workgroups of 8 wavefronts in two key groups, combined through LDS (prefetch depth 1, 2;
 *                       13 is chosen when there is at most one 128-row workgroup per CU);
 *                   15 = software-pipelined 128-row workgroups (d = 128; softmax of one key tile woven between the MFMAs
 *                       of the next).
 *   "attn_split"    0 = the library decides whether several workgroups share the keys of a row tile (default: only with at
 *                   most 128 workgroups and at least 32 key tiles, and only when the call brings the workspace);
 *                   1 = never; 2..16 = that many (lowered to keep four key tiles per workgroup).
 *   "lmhead_variant" -1 = pick the LM-head kernel shape (workgroup tile, wavefront layout, prefetch depth) from M
 *                   (default); >= 0 forces one entry of the library's shape table.
 *   "lmhead_block"  -1 = automatic blocking of LM-head workgroups per XCD (default); 0 = none (row chunks of one
 *                   vocabulary tile side by side); 1..8 = that many vocabulary tiles per block.
 *   "lmhead_nt"     1 = when a launch has one row chunk (every element of W used once) fetch W with non-temporal
 *                   loads (default); 0 = never.
 *   "lmhead_cus"    0 = the half-height tail rule of the LM head assumes the device's CU count (default); n > 0 = assume n
 *                   (tests: makes a small vocabulary take the two-launch path); -1 = no half-height tail.
 *   "attn_nt"       1 = non-temporal K/V loads when one workgroup is the only reader of its (sequence, KV head)
 *                   (g*Lq <= 32; default); 0 = never.
 *   "kv_copy_unroll" 16-byte pieces per thread of the copy kernel (1, 2, 4 or 8), plus 16 when K and V are copied by
 *                   different workgroups, plus 32 / 64 for non-temporal loads / stores (default: 17).
 *   "attn_remap"    bit mask, default 7: 1 = 128-row workgroups of one (sequence, KV head) run on ONE XCD (1-D
 *                   grid; forward and the dQ pass), 2 = under a block-causal mask the row tile with the longest
 *                   key range is dispatched first, 4 = the same grouping for the dK / dV passes; 0 = plain
 *                   (tile, KV head, sequence) grids.
 * The knobs exist for tests and tuning sweeps. */
int dlm_set_option(const char *name, int value);

const char *dlm_last_error(void);
int dlm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DLM_H */
