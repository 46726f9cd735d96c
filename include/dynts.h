/*
 * dynts.h -- C ABI of the MI355X (gfx950) DynTS decode hot path.
 *
 * DynTS (Dynamic Thinking-Token Selection) decodes over a budget-bounded KV cache: per
 * layer the cache of a sequence is the question window (M prompt slots, never evicted),
 * the selection window and the local window (Sec. 4.2).  Every decode step attends over
 * the retained slots (Eq. attn-score, Eq. attn-o), every cached thinking token carries an
 * importance score (Eq. importance-score, kept here in running form per layer and KV
 * head), and on a trigger the top-k thinking tokens of the selection window are kept and
 * the rest evicted.
 *
 * Conventions
 *  - All array arguments are DEVICE pointers unless a comment says "host".  The caller
 *    owns every buffer; the context owns host metadata only and never allocates device
 *    memory.  bf16 arrays are passed as uint16_t (raw bits).
 *  - Every call enqueues its kernels on the caller's stream (a hipStream_t passed as
 *    void*, NULL = the null stream) and returns without synchronising the host.  Calls on
 *    one context must be stream-ordered with respect to each other.
 *  - Return value: DYNTS_OK or a negative error.  Argument errors are found on the host
 *    before anything is launched.  Conditions only the device can see (a sequence that
 *    would overflow `capacity`) are latched into the bound `status` word: bit 0 = an
 *    append was dropped because the cache was full; bit 1 (value 2) = keep_idx too short for a sequence
 *    (dynts_select_evict left it alone); bit 2 (value 4) = the page pool of the paged layout ran dry.
 *  - Layout (C order, L = n_layers, Nb = batch, Hkv = n_kv_heads, cap = capacity, d = head_dim):
 *      K, V      bf16  [L][Nb][Hkv][cap][d]   rows in position order
 *      S         fp32  [L][Nb][Hkv][cap]      importance score; +inf on question slots
 *      pos       int32 [L][Nb][Hkv][cap]      original token position of each slot
 *      seq_len   int32 [L][Nb]                slots in use (equal for all KV heads)
 *      next_pos  int32 [L][Nb]                position the next appended token receives
 *      n_prompt  int32 [Nb]                   M of each sequence
 *  - Query head hq reads KV head hq / G, G = n_q_heads / n_kv_heads (grouped-query
 *    attention, Sec. 2 "Attention Mechanism").  Supported: head_dim 64 or 128, G <= 16.
 *  - `active` (uint8 [Nb], may be NULL = all active) masks finished sequences of a ragged
 *    batch: nothing is appended, attended or written for them.
 */
#ifndef DYNTS_H
#define DYNTS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DYNTS_OK 0
#define DYNTS_EINVAL (-1)     /* a value outside its documented range */
#define DYNTS_ENULL (-2)      /* a required pointer is NULL */
#define DYNTS_ESHAPE (-3)     /* unsupported shape: head_dim, group size, divisibility */
#define DYNTS_ECAPACITY (-4)  /* capacity < budget + window + evict_every, or an index stride too small */
#define DYNTS_ENOTBOUND (-5)  /* dynts_bind has not been called */
#define DYNTS_EWORKSPACE (-6) /* workspace smaller than dynts_workspace_bytes, or misaligned */
#define DYNTS_EHIP (-7)       /* the HIP runtime refused a launch */
#define DYNTS_EPENDING (-8)   /* rows would move while a score update is still deferred */

#define DYNTS_SCORE_ACCUMULATE 0 /* score = attention received so far (Eq. importance-score) */
#define DYNTS_SCORE_EXTERNAL 1   /* score supplied at append (the predictor's output, Sec. 4.1) */

typedef struct dynts_config {
  int32_t n_layers;
  int32_t batch;
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t head_dim;
  int32_t capacity;     /* cap: slots per (sequence, KV head); >= prompt + budget + window + evict_every, <= 2^22 */
  int32_t budget;       /* selection-window slots kept by a trigger (the k of top-k, default k_keep) */
  int32_t window;       /* local-window slots, always kept */
  int32_t evict_every;  /* trigger period in steps = eviction volume K of Sec. 5 */
  float softmax_scale;  /* 0 => 1/sqrt(head_dim) (Eq. attn-score) */
  int32_t score_mode;   /* DYNTS_SCORE_* */
} dynts_config;

typedef struct dynts_ctx dynts_ctx;

/* Library version, major*10000 + minor*100 + patch. */
int dynts_version(void);
/* Static text for an error code. */
const char *dynts_strerror(int code);

/* Validate `cfg` and make a host-side context.  No device work, no HIP call. */
int dynts_create(const dynts_config *cfg, dynts_ctx **out);
int dynts_destroy(dynts_ctx *ctx);

/* Bytes of device scratch the kernels need for `cfg` (split partials, the saved query and
 * softmax statistics of the deferred score update).  0 if cfg is invalid. */
size_t dynts_workspace_bytes(const dynts_config *cfg);

/* Launch shape of the attention kernel, for tuning and for tests that must reach a particular shape at a
 * small size: the cache of a (sequence, KV head) is split over about target_workgroups / (batch * n_kv_heads)
 * workgroups (at least one; 0 = the default, one workgroup per compute unit) of waves_per_workgroup waves
 * (4 or 8; 0 = the default, 8).  Results do not depend on the shape beyond rounding order.  Changes the
 * workspace layout: call it before dynts_bind (it unbinds), and size the workspace with
 * dynts_ctx_workspace_bytes. */
int dynts_set_launch_shape(dynts_ctx *ctx, int32_t target_workgroups, int32_t waves_per_workgroup);
/* Bytes of workspace this context needs (= dynts_workspace_bytes(cfg) unless the launch shape was changed). */
size_t dynts_ctx_workspace_bytes(const dynts_ctx *ctx);

/* Attach the caller's device buffers (layout above).  `workspace` must be 256-byte aligned
 * and zero-filled once by the caller before first use; `status` is one int32, zeroed by
 * the caller.  Binding resets the context's deferred-update bookkeeping. */
int dynts_bind(dynts_ctx *ctx, uint16_t *K, uint16_t *V, float *S, int32_t *pos,
               int32_t *seq_len, int32_t *next_pos, int32_t *n_prompt, void *workspace,
               size_t workspace_bytes, int32_t *status);

/* Paged (block-table) layout instead of one dense [cap][d] array per unit: K_pool, V_pool bf16
 * [n_pages][64][d] hold the rows of ALL layers, sequences and KV heads; slot j of a unit is row j % 64 of page
 * block_table[layer][b][h][j / 64] (int32 [L][Nb][Hkv][max_pages], max_pages * 64 >= capacity).  Pages are taken
 * from and returned to a device-side free stack: free_stack int32 [n_pages] lists page ids, *free_top (device
 * int32) is the number of free ones (entries [0, *free_top) are free).  The caller initialises the stack (all
 * pages free: free_stack[i] = i, *free_top = n_pages) and leaves the block table alone; appends and
 * dynts_prefill pop, dynts_compact gives the pages past the new length back, so evicted memory can be taken by
 * any other sequence.  dynts_prefill expects the layer's units to hold no pages.  When the stack runs dry the
 * row is dropped and bit 2 (value 4) of the status word is latched; results are undefined from then on.
 * The pools must hold finite values before first use (zero-filled, say): rows beyond a sequence's length may be
 * read, with zero weight.  S, pos and the per-sequence arrays keep the dense layout.  Everything else behaves as after dynts_bind.
 * The ORDER of the ids in the initial stack is the caller's choice and decides where a unit's pages lie.  With ids in
 * order, sequences that append in step get neighbouring pages round after round, so a unit's pages lie a fixed
 * power-of-two stride apart: good for caches streamed from HBM, but a cache small enough to stay in the 256 MB
 * memory-side cache then runs up to 25 % slower than with a shuffled stack (measured, 159 MB of K/V: 35 - 40 us per
 * attend launch in order, 31.5 us shuffled, 30 us dense); beyond that size a shuffled stack costs 3 - 5 %. */
int dynts_bind_paged(dynts_ctx *ctx, uint16_t *K_pool, uint16_t *V_pool, int32_t n_pages, int32_t *block_table,
                     int32_t max_pages, int32_t *free_stack, int32_t *free_top, float *S, int32_t *pos,
                     int32_t *seq_len, int32_t *next_pos, int32_t *n_prompt, void *workspace,
                     size_t workspace_bytes, int32_t *status);

/* Question window (Sec. 4.2, first paragraph): copy the prompt rows of one layer,
 * K0, V0 bf16 [Nb][Hkv][m_max][d], m int32 [Nb] with m[b] <= m_max, into slots [0, m[b]);
 * scores +inf, pos = slot, seq_len = next_pos = n_prompt = m. */
int dynts_prefill(dynts_ctx *ctx, int32_t layer, const uint16_t *K0, const uint16_t *V0,
                  int32_t m_max, const int32_t *m, void *stream);

/* Append the current token (Sec. 4.2, second paragraph): k_new, v_new bf16 [Nb][Hkv][d] go
 * to slot seq_len[b] of every KV head; score 0, or s_new fp32 [Nb][Hkv] when score_mode is
 * DYNTS_SCORE_EXTERNAL (then s_new is required); pos = next_pos++; seq_len++. */
int dynts_append(dynts_ctx *ctx, int32_t layer, const uint16_t *k_new, const uint16_t *v_new,
                 const float *s_new, const uint8_t *active, void *stream);

/* Decode attention (Eq. attn-score, Eq. attn-o): for each active sequence and query head,
 * out[b][hq][:] = sum_j softmax_j(q.k_j * scale) v_j over slots [0, seq_len[b]).
 * q bf16 [Nb][Hq][d]; out fp32 [Nb][Hq][d]; lse fp32 [Nb][Hq] (may be NULL) receives
 * log sum_j exp(logit_j).  Leaves what dynts_update_scores needs in the workspace. */
int dynts_decode_attend(dynts_ctx *ctx, int32_t layer, const uint16_t *q, const uint8_t *active,
                        float *out, float *lse, void *stream);

/* Score accumulation (Eq. importance-score in running form; App. B.1 sums over heads):
 * S[b][h][j] += sum over the G heads of the group of alpha[g][j], for every thinking slot
 * j >= n_prompt[b] the last attend call of this layer saw.  A no-op when nothing is
 * outstanding or score_mode is external. */
int dynts_update_scores(dynts_ctx *ctx, int32_t layer, void *stream);

/* dynts_decode_attend with the score accumulation fused into the same pass over K: the
 * accumulation owed by the PREVIOUS attend call of this layer is applied while this call
 * streams the cache, and this call's own accumulation becomes the outstanding one.  S
 * therefore lags by one step until dynts_update_scores (or dynts_select_evict, which
 * applies it first) is called. */
int dynts_decode_attend_update(dynts_ctx *ctx, int32_t layer, const uint16_t *q,
                               const uint8_t *active, float *out, float *lse, void *stream);

/* One whole decode step of a layer in one pass: dynts_append + dynts_decode_attend_update.  A sequence whose
 * cache is already full is left alone in this step (nothing appended, attended or scored; status bit 0). */
int dynts_decode_step(dynts_ctx *ctx, int32_t layer, const uint16_t *q, const uint16_t *k_new,
                      const uint16_t *v_new, const float *s_new, const uint8_t *active,
                      float *out, float *lse, void *stream);

/* dynts_decode_step for callers that cannot allocate device memory and want to hand over as little as possible
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same step, but
 * the launch's scratch -- the split partials and the ticket counters, i.e. everything in the workspace that
 * does not have to survive the call -- lives in an array that is part of the library's code object on each
 * GPU (DYNTS_STATIC_SCRATCH_BYTES = 8 MiB, held until the process ends) instead of the head of the
 * bound workspace.  The call allocates nothing and frees nothing, on the host side of HIP or the device side.
 * The state that carries over between steps (saved queries and softmax statistics of the deferred score
 * update) stays in the bound workspace, so this call and dynts_decode_step may be mixed freely on a context.
 *  - DYNTS_EWORKSPACE if the context's shape needs more scratch than the array holds: the partials take
 *    batch * n_kv_heads * chunks * group * (head_dim + 2) * 8 bytes of its upper 7 MiB (chunks being what
 *    dynts_set_launch_shape describes; with the default shape 2 MiB on the 32-sequence Qwen-shaped workload,
 *    nothing once there are as many (sequence, KV head) units as compute units), the counters 4 bytes per
 *    unit and per sequence of 512 KiB each.  Nothing is launched then.
 *  - All calls on one GPU share that GPU's array, from every context and stream: calls that may overlap in
 *    time on one GPU race with each other -- keep them on one stream or order them with events.  (Calls that
 *    are stream-ordered leave the array as the next one needs it, whatever its shape: counters live in a part
 *    of the array that holds nothing else and are back at zero when a launch ends, partials are tagged with
 *    a serial number that no other launch of the process uses.)
 *  - The first call on a GPU looks the array up and clears it with a small kernel on the caller's stream. */
#define DYNTS_STATIC_SCRATCH_BYTES (8u << 20)
int dynts_decode_step_static(dynts_ctx *ctx, int32_t layer, const uint16_t *q, const uint16_t *k_new,
                             const uint16_t *v_new, const float *s_new, const uint8_t *active,
                             float *out, float *lse, void *stream);

/* Optional announcement: the next fused step of this layer (dynts_decode_step, dynts_decode_step_static or
 * dynts_decode_attend_update) will be followed by a trigger (dynts_select_evict).  That step then keeps its
 * logits (4 bytes per slot and query head of the group, in the workspace), and the score accumulation it owes
 * is applied from them when dynts_select_evict / dynts_update_scores asks for it, instead of by a second pass
 * over K.  Results are the same up to fp32 rounding order; without the announcement everything works as before.
 * dynts_decode_loop makes it itself on the steps flagged in evict_steps.  No effect with external scores. */
int dynts_hint_trigger(dynts_ctx *ctx, int32_t layer);

/* KV-cache selection (Sec. 4.2, third paragraph): for every sequence with trigger[b] != 0
 * (uint8 [Nb], NULL = all) and every KV head keep all question slots, the last `window`
 * slots, and of the slots between them the k_keep with the highest score (ties: lower
 * position first -- decided by SLOT order: the kernel never reads `pos`, it relies on the
 * invariant that slots are in position order, which appends and the stable compaction keep).  keep_idx int32 [Nb][Hkv][keep_stride] receives the retained slots in
 * ascending order, new_len int32 [Nb] their count (seq_len[b] where not triggered or when
 * the selection window holds <= k_keep slots).  k_keep < 0 means cfg.budget.  Applies an
 * outstanding score accumulation first.  NaN scores give an unspecified (in-bounds) choice. */
int dynts_select_evict(dynts_ctx *ctx, int32_t layer, const uint8_t *trigger, int32_t k_keep,
                       int32_t *keep_idx, int32_t keep_stride, int32_t *new_len, void *stream);

/* Eviction (Sec. 4.2): stable in-place gather of the K, V, S and pos rows listed in
 * keep_idx to slots [0, new_len[b]) and seq_len[b] = new_len[b], for triggered sequences.
 * keep_idx rows must be strictly ascending and < seq_len[b] (indices are clamped into the
 * cache, never followed out of bounds).  DYNTS_EPENDING if a score accumulation is
 * outstanding for this layer. */
int dynts_compact(dynts_ctx *ctx, int32_t layer, const uint8_t *trigger, const int32_t *keep_idx,
                  int32_t keep_stride, const int32_t *new_len, void *stream);

/* Native decode loop: enqueue n_steps whole steps of every layer without returning to the
 * caller -- per step and layer dynts_decode_step, and on steps with evict_steps[i] != 0
 * (host uint8 [n_steps]) dynts_select_evict(k_keep = budget) + dynts_compact for the
 * sequences flagged in trigger (device uint8 [n_steps][Nb], NULL = all).
 *   q      bf16 [n_steps][L][Nb][Hq][d]      k_new, v_new bf16 [n_steps][L][Nb][Hkv][d]
 *   s_new  fp32 [n_steps][Nb][Hkv] (external mode, same score for every layer) or NULL
 *   active uint8 [n_steps][Nb] or NULL
 *   out    fp32 [L][Nb][Hq][d], overwritten every step (out_step_stride = 0) or one slab
 *          per step (out_step_stride = L*Nb*Hq*d elements)
 *   keep_idx int32 [Nb][Hkv][cap], new_len int32 [Nb]: scratch for the triggers. */
int dynts_decode_loop(dynts_ctx *ctx, int32_t n_steps, const uint16_t *q, const uint16_t *k_new,
                      const uint16_t *v_new, const float *s_new, const uint8_t *active,
                      const uint8_t *evict_steps, const uint8_t *trigger, float *out,
                      size_t out_step_stride, int32_t *keep_idx, int32_t *new_len, void *stream);

/* Measurement hook: when both are non-NULL hipEvent_t handles (created by the caller with
 * timing enabled), every later attend launch of this context attaches them to the dispatch
 * of its streaming kernel (attention + deferred score update, the kernel that moves the K/V
 * bytes): `start` is stamped when that kernel begins, `stop` when it ends, so
 * hipEventElapsedTime(start, stop) is the kernel's own duration.  Pass NULLs to switch it off. */
int dynts_set_kernel_events(dynts_ctx *ctx, void *start, void *stop);

/* The same for a run of launches: `starts` and `stops` are host arrays of n hipEvent_t handles; the
 * next n attend launches of this context (in call order, e.g. inside dynts_decode_loop) take one pair
 * each, after which the hook is off again.  n = 0 clears the list. */
int dynts_set_kernel_event_list(dynts_ctx *ctx, void *const *starts, void *const *stops, int32_t n);

/* Importance score from a block of queries at once (Eq. importance-score with its sum over the K
 * answer tokens; App. B.1: the answer-by-thinking sub-matrix of the attention weights summed over
 * heads and over the answer dimension):
 *   dst[b][h][j] (+)= sum over the n_queries block queries i and the G heads g of the group of
 *                    alpha_{(i,g), j},   for the cached slots j < seq_len[b],
 * where query i's softmax (Eq. attn-score) runs over the cached slots and, when k_blk is given, over
 * block keys 0..i (causal, as in one forward pass over the block; block tokens receive no score).
 *   q_blk bf16 [Nb][n_queries][Hq][d]     k_blk bf16 [Nb][n_queries][Hkv][d] or NULL
 *   dst fp32 [Nb][Hkv][cap]: every slot j < seq_len[b] is written (question slots too).  dst = NULL
 *     means the layer's score array S; then slots below n_prompt[b] keep their +inf.
 *   accumulate != 0 adds to dst, 0 overwrites it.
 *   scratch: >= dynts_score_block_scratch_bytes(cfg, n_queries) bytes of device memory, 4-byte
 *     aligned, contents irrelevant before and after.
 * Independent of the deferred accumulation of the fused decode calls (sums commute).  The cache is
 * only read. */
size_t dynts_score_block_scratch_bytes(const dynts_config *cfg, int32_t n_queries);
int dynts_score_block(dynts_ctx *ctx, int32_t layer, const uint16_t *q_blk, const uint16_t *k_blk,
                      int32_t n_queries, const uint8_t *active, float *dst, int32_t accumulate,
                      void *scratch, size_t scratch_bytes, void *stream);

/* Importance Predictor (Sec. 4.1; App. A "Predictor Overhead", App. C for the sizes): the three-layer
 * MLP d -> m1 -> m2 -> 1 on the final hidden state of the current token,
 *   s[b] = w3 . act(W2 act(W1 h[b] + b1) + b2) + b3,
 * whose output is the score the paper's inference mode appends with the token (dynts_append / dynts_decode_step
 * with score_mode DYNTS_SCORE_EXTERNAL take it as s_new).  Weights are device pointers, bf16 row-major
 * [out][in]; biases fp32 or NULL.  The paper calls the MLP "linear" and names no activation: it is a
 * parameter.  Products are accumulated in fp32 and nothing is rounded to bf16 between the layers.
 *   h bf16 [batch][d], batch <= 128;  d and m1 multiples of 32, m2 a multiple of 16.
 *   s_out fp32 [batch][n_rep]: the score of sequence b written n_rep times (n_rep = n_kv_heads gives the
 *     [Nb][Hkv] layout of s_new: one score per token for every head, as in the paper).
 *   scratch: >= dynts_predict_scratch_bytes bytes, 256-byte aligned, zero-filled once by the caller before its
 *     first use (it may be shared by calls that are stream-ordered with respect to each other).
 *   start/stop: optional hipEvent_t handles attached to the first and the last kernel of the call. */
#define DYNTS_ACT_NONE 0
#define DYNTS_ACT_RELU 1
#define DYNTS_ACT_SILU 2
typedef struct dynts_predictor {
  int32_t d, m1, m2;
  int32_t activation; /* DYNTS_ACT_* */
  int32_t packed;     /* 0: W1, W2 row-major [out][in]; 1: both in the tiled layout of dynts_predictor_pack */
  const uint16_t *W1; /* [m1][d] */
  const float *b1;    /* [m1] or NULL */
  const uint16_t *W2; /* [m2][m1] */
  const float *b2;    /* [m2] or NULL */
  const uint16_t *w3; /* [m2] */
  const float *b3;    /* [1] or NULL */
} dynts_predictor;
/* One-off repacking of a row-major bf16 weight matrix W [m][K] (m a multiple of 16, K of 32) into tiles of
 * 16 rows x 32 columns stored contiguously, W_packed [m/16][K/32][16][32] (same size, must not alias W).
 * With packed weights every load instruction of the GEMM reads one contiguous kilobyte instead of 16 pieces a
 * whole weight row apart, which is what lets the weight stream run at memory speed. */
int dynts_predictor_pack(const uint16_t *W, int32_t m, int32_t K, uint16_t *W_packed, void *stream);
size_t dynts_predict_scratch_bytes(const dynts_predictor *w, int32_t batch);
int dynts_predict_scores(const dynts_predictor *w, const uint16_t *h, int32_t batch, float *s_out,
                         int32_t n_rep, void *scratch, size_t scratch_bytes, void *start, void *stop,
                         void *stream);

/* Measurement aid, not part of the method: one launch of a plain read stream over `bytes` (a multiple
 * of 16, buf 16-byte aligned) of device memory, 16 bytes per lane per load, n_workgroups x 256 lanes,
 * grid-stride.  Nothing is written unless the XOR of all words equals `magic` (then sink[0], one
 * device uint32, receives it).  start/stop: hipEvent_t handles attached to the dispatch as in
 * dynts_set_kernel_events, or both NULL.  Its rate on a buffer of the cache's size is the bandwidth
 * the simplest kernel reaches, to set beside the published peak. */
int dynts_probe_read_stream(const void *buf, size_t bytes, int32_t n_workgroups, uint32_t magic,
                            uint32_t *sink, void *start, void *stop, void *stream);

/* Measurement aid, not part of the method: one launch in which every lane of n_workgroups x 256 lanes performs
 * iters x 8 exponentials 2^x followed by a subtraction (the loop holds nothing else), 16 * iters instructions per
 * wave.  The exponentials delivered per second are the second roofline of dynts_score_block, which needs one
 * per (query row, slot) and pass (Eq. attn-score's softmax).  sink: one device float, written only on a value
 * that cannot occur.  start/stop: hipEvent_t handles attached to the dispatch, or both NULL. */
int dynts_probe_exp_rate(int32_t n_workgroups, int32_t iters, float *sink, void *start, void *stop, void *stream);

/* Measurement aid, not part of the method: the instruction mix of dynts_score_block's kernels with no memory
 * access.  Every wave of n_workgroups x 256 lanes runs iters rounds of what one streamed 16-row tile costs it
 * there: what & 1: 16 bf16 MFMAs (16x16x32) on four independent accumulators; what & 2: 16 x (multiply-add, 2^x,
 * add) on independent registers; what = 3: both, interleaved by the compiler as in the kernels.  The time per
 * round and SIMD is the floor of a tile that instruction issue and the two pipes set (Eq. attn-score's softmax
 * needs the three vector instructions per logit).  sink, start/stop as for dynts_probe_exp_rate. */
int dynts_probe_issue_mix(int32_t n_workgroups, int32_t iters, int32_t what, float *sink, void *start, void *stop,
                          void *stream);

#ifdef __cplusplus
}
#endif
#endif /* DYNTS_H */
