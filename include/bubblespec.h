/*
 * bubblespec.h -- C ABI of the speculative-verification decode step for AMD MI355X (gfx950).
 *
 * The step is the inner loop of the paper's rollout procedure (Alg. 1): retrieve a block of
 * draft tokens for every running sequence from that prompt's pool of pre-generated rollouts
 * (Sec. 3.2), run the target decoder once over the k+1 positions [last token, draft_1..draft_k]
 * of every sequence (Sec. 3.3: token-wise linear/norm operations plus one "unified" attention
 * launch that serves every query length 1..k_max+1 in the same batch), accept or reject the
 * drafts by the exact rule of Eq. 2-3, and keep the accepted prefix in the KV cache.
 *
 * Conventions
 *   - Plain C.  Every call returns bs_status; nothing throws or aborts.
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are ordinary host memory.
 *   - OWNERSHIP: the caller allocates and owns every device buffer (weights, KV pages, block
 *     table, context lengths, pool, workspace, inputs, outputs).  The library owns only the
 *     host-side bs_ctx; it never allocates or frees device memory.
 *   - `stream` is a hipStream_t passed as void*.  Step calls only enqueue work on it and never
 *     synchronise with the host.  Conditions only the device can see (a sequence running past
 *     its pages, a token id outside the vocabulary, a draft length above k_max) set bits in a
 *     device status word; the affected sequence is skipped (no row of it is embedded, appended,
 *     judged or committed: n_accepted = n_emitted = 0, out_tokens = -1, ctx_len unchanged), nothing
 *     is written out of bounds, and bs_poll_status() (the one synchronising call) returns the word.
 *   - Row packing: sequence b contributes k_b+1 query rows; rows are packed in batch order,
 *     row0_b = sum_{b'<b}(k_b'+1), M = sum_b (k_b+1).  Draft rows (for q_logits) are packed the
 *     same way with k_b rows per sequence, T_d = sum_b k_b.  The packing is computed on the
 *     device from draft_len, so draft_len may itself be the output of bs_draft_lookup.
 */
#ifndef BUBBLESPEC_H
#define BUBBLESPEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  BS_OK = 0,
  BS_EINVAL = 1,    /* null pointer, bad enum, bad scalar */
  BS_ESHAPE = 2,    /* sizes inconsistent with the model / B_max / k_max */
  BS_ECAPACITY = 3, /* workspace too small, KV description cannot hold the request */
  BS_ESTATE = 4,    /* call order violated (e.g. accept before verify, lookup before pool_bind) */
  BS_EHIP = 5       /* a HIP runtime call failed; see bs_last_error */
} bs_status;

typedef enum { BS_F32 = 0, BS_BF16 = 1 } bs_dtype;

/* bits of the device status word returned by bs_poll_status */
enum {
  BS_FAULT_DRAFT_LEN = 1, /* draft_len[b] outside [0, k_max]                      */
  BS_FAULT_KV_PAGES = 2,  /* c_b + k_b + 1 exceeds the pages of the slot / bad page id */
  BS_FAULT_TOKEN_ID = 4,  /* a token id outside [0, vocab)                         */
  BS_FAULT_COMMIT = 8,    /* n_commit[b] outside [0, k_b + 1]                      */
  BS_FAULT_SLOT = 16,     /* seq_slot[b] outside [0, n_slots) or used twice        */
  BS_FAULT_RANGE = 32     /* bf16 models: a value left the float16 range (see bs_model_desc.dtype) and was
                             saturated; the step's results are finite but no longer those of the model */
};

#define BS_PAGE_TOKENS 64 /* tokens per KV page (fixed) */
#define BS_MAX_K 30       /* largest supported k_max (near_tie is a 32-bit mask) */

/* Decoder shape.  The paper treats the target policy as a black box (Sec. 4.1 uses Qwen-family
 * decoders); this is the pre-norm RMSNorm / rotary (rotate-half pairing) / GQA / SwiGLU decoder
 * with an untied LM head and no biases. */
typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  int32_t dtype;   /* bs_dtype of the weights and of the KV cache (data at rest).  BS_BF16 models compute with
                      float16 matrix operands and float32 accumulation: weights and cached K/V are bf16 VALUES
                      held in float16 encoding (exact for 6.1e-5 <= |x| <= 65504, smaller magnitudes lose low
                      bits), activations between operators are float16, the residual stream is float32.  Any
                      weight, K/V element or activation with |x| > 65504 (or NaN) is saturated to +-65504 (NaN
                      to 0) and reported through BS_FAULT_RANGE; nothing infinite enters a matrix product. */
  float rms_eps;   /* RMSNorm epsilon */
  float rope_theta;
} bs_model_desc;

/* Weights: device pointers, row-major [out_features, in_features] (so y = W x), dtype =
 * desc.dtype, except the norm gains which are always float32.  The per-layer members are HOST
 * arrays of n_layers device pointers (copied at bs_create; the arrays need not outlive it). */
typedef struct {
  const void* embed;               /* dev [vocab, d_model]                              */
  const void* lm_head;             /* dev [vocab, d_model]                              */
  const float* final_norm;         /* dev [d_model]                                     */
  const float* const* attn_norm;   /* host[L] -> dev [d_model]                          */
  const void* const* wqkv;         /* host[L] -> dev [(Hq+2*Hkv)*D, d_model]: q,k,v rows */
  const void* const* wo;           /* host[L] -> dev [d_model, Hq*D]                    */
  const float* const* mlp_norm;    /* host[L] -> dev [d_model]                          */
  const void* const* w_gate_up;    /* host[L] -> dev [2*d_ffn, d_model]: gate rows, then up rows */
  const void* const* w_down;       /* host[L] -> dev [d_model, d_ffn]                   */
} bs_weights;

/* Paged KV cache.  A page holds BS_PAGE_TOKENS tokens of one layer for all KV heads.  The page
 * byte size is Hkv * BS_PAGE_TOKENS * D * sizeof(dtype), for K and for V.  Element order and
 * encoding inside a page are private to the library (bf16 models: matrix-unit operand order, each
 * bf16-rounded value held as IEEE float16 bits, which is exact for 6.1e-5 <= |x| <= 65504); use
 * bs_kv_write / bs_kv_read to move dense rows (in desc.dtype) in and out.
 *   block_table[slot][j] = page id of tokens [j*64, j*64+64) of that slot (same id in all layers)
 *   ctx_len[slot]        = committed length c of the slot; advanced only by bs_kv_commit.
 * Pages must hold finite values before first use (zero-fill them once): positions beyond a row's
 * causal limit enter the P*V product with weight exactly 0, and 0 * NaN would still poison it. */
typedef struct {
  int32_t n_pages, n_slots, max_pages_per_seq;
  void* const* k_pages;   /* host[L] -> dev [n_pages] pages */
  void* const* v_pages;   /* host[L] -> dev [n_pages] pages */
  const int32_t* block_table; /* dev [n_slots, max_pages_per_seq] */
  int32_t* ctx_len;           /* dev [n_slots] */
} bs_kv_desc;

typedef struct bs_ctx bs_ctx;

/* Bytes of device workspace a context for (desc, B_max, k_max) needs. 0 on invalid arguments. */
size_t bs_workspace_bytes(const bs_model_desc* desc, int B_max, int k_max);

/* Creates the host-side context.  `workspace` (dev, 256-byte aligned, >= bs_workspace_bytes)
 * stays owned by the caller and must outlive the context.  Enqueues on `stream` a clear of the
 * device status word and, for bf16 models, a one-time re-pack of the projection and LM-head
 * matrices into the workspace (float16, matrix-unit operand order); after that work has finished
 * the library no longer reads wqkv / wo / w_gate_up / w_down / lm_head (embed and the norm gains
 * are still read in place).  Errors: BS_EINVAL (null / bad dtype), BS_ESHAPE (unsupported shape: head_dim
 * not in {64,128}, d_model or d_ffn not a multiple of 64, d_model > 16384, Hq % Hkv != 0,
 * k_max > BS_MAX_K, bf16 models with (k_max+1) * Hq/Hkv > 128),
 * BS_ECAPACITY (workspace too small). */
bs_status bs_create(const bs_model_desc* desc, const bs_weights* weights, const bs_kv_desc* kv,
                    void* workspace, size_t workspace_bytes, int B_max, int k_max, void* stream,
                    bs_ctx** out);
void bs_destroy(bs_ctx* ctx);
/* Static, human-readable description of the last non-OK status of this context. */
const char* bs_last_error(const bs_ctx* ctx);

/* Sec. 3.2: binds the draft database.  Rollouts are stored back to back in pool_tokens;
 * rollout r is pool_tokens[rollout_offsets[r] .. rollout_offsets[r+1]); prompt p owns rollouts
 * prompt_rollout_begin[p] .. prompt_rollout_begin[p+1].  All three arrays are dev and stay owned
 * by the caller.  n_rollouts is the total rollout count.  BS_EINVAL on null / negative sizes. */
bs_status bs_pool_bind(bs_ctx* ctx, int n_prompts, int n_rollouts, const int32_t* pool_tokens,
                       const int64_t* rollout_offsets, const int32_t* prompt_rollout_begin);

/* Sec. 3.2: prebuilt draft index (the per-prompt suffix structure with occurrence counts).  bs_index_build
 * runs on the HOST: all three arrays are host pointers with the layout of bs_pool_bind; it returns a
 * library-owned, position-independent blob (*blob_out, *bytes_out; release with bs_index_free).  The caller
 * copies the blob to device memory and binds both copies with bs_index_bind (the host copy is only read during
 * the call, the device copy must stay valid while bound; NULL, NULL unbinds).  While an index is bound
 * bs_draft_lookup walks it (O(max_match + k_max) dependent loads per sequence) instead of scanning the pool,
 * and returns exactly the same drafts.  Errors: BS_EINVAL (null, negative token, inconsistent offsets, foreign
 * blob), BS_ESHAPE (a prompt's pool beyond 2^29 tokens), BS_ECAPACITY (out of host memory). */
bs_status bs_index_build(int n_prompts, const int32_t* pool_tokens /*host*/, const int64_t* rollout_offsets /*host*/,
                         const int32_t* prompt_rollout_begin /*host*/, void** blob_out /*host*/, size_t* bytes_out);
void bs_index_free(void* blob);
bs_status bs_index_bind(bs_ctx* ctx, const void* blob_host, const void* blob_dev, size_t bytes);

/* Sec. 3.2 / Alg. 1 "retrieve a draft block": for each sequence b, match the last m tokens of
 * its rollout (tail_tokens[b], newest last, entries < 0 are padding) against the pool of prompt
 * seq_prompt[b], m from max_match down to min_match, taking the first m that occurs; then walk
 * up to k_max continuation tokens, each time taking the token that follows the most occurrences
 * (ties: smaller id) and keeping only the occurrences it follows.  Occurrences never straddle
 * rollouts.  Output draft_len[b] in [0,k_max]; draft_tokens[b][i >= draft_len[b]] = -1.
 * All pointers dev.  Errors: BS_ESTATE (no pool or index bound), BS_ESHAPE (B > B_max, k_max > ctx k_max,
 * max_match outside [1,8], min_match outside [1,max_match]), BS_EINVAL (null). */
bs_status bs_draft_lookup(bs_ctx* ctx, int B, const int32_t* seq_prompt /*[B]*/,
                          const int32_t* tail_tokens /*[B,max_match]*/, int max_match, int min_match,
                          int k_max, int32_t* draft_tokens /*[B,k_max]*/, int32_t* draft_len /*[B]*/,
                          void* stream);

/* Sec. 3.3 / Alg. 1 "p_t under prefix y" for all t at once: one forward pass of the decoder over
 * rows [last_token[b], draft_tokens[b][0..k_b)] at positions c_b .. c_b+k_b, where c_b =
 * ctx_len[seq_slot[b]].  Side effects: K/V rows of those positions are written (tentatively) to
 * the slot's pages in every layer; the final-norm hidden rows are kept in the workspace for
 * bs_accept_resample.  ctx_len is NOT changed.  logits_debug, if not NULL, receives the float32
 * logits of all rows, packed [M, vocab] (caller sizes it for B*(k_max+1) rows).
 * All pointers dev.  Errors: BS_EINVAL, BS_ESHAPE (B > B_max or k_max > ctx k_max). */
bs_status bs_verify_step(bs_ctx* ctx, int B, const int32_t* seq_slot /*[B]*/,
                         const int32_t* last_token /*[B]*/, const int32_t* draft_tokens /*[B,k_max]*/,
                         const int32_t* draft_len /*[B]*/, int k_max, float* logits_debug,
                         void* stream);

/* Eq. 2-3 / Alg. 1 accept loop on the rows of the preceding bs_verify_step (same B, k_max,
 * draft arrays).  p_i = softmax(z_i / temperature) (temperature 0: one-hot at the first arg-max).
 * q_logits == NULL selects the paper's deterministic proposal (accept draft i+1 with probability
 * p_i(draft)); otherwise q_i = softmax(q_logits row) and the general rule min(1, p/q) /
 * max(0, p - q) is applied.  Accept iff u_accept[b][i] < min(1, rho).  One token per sequence is
 * sampled with u_sample[b] by inverse CDF in vocabulary order (float64 running sum): the recovered
 * token at the first rejection, or the bonus token after full acceptance (if emit_bonus), or the
 * plain sample when k_b == 0.  An accepted eos_id (>= 0) ends the block.
 * Outputs: n_accepted[b]; out_tokens[b][0..n_emitted[b]) = accepted drafts then the sampled token
 * (rest -1); near_tie[b]: bit i set if |rho_i - u_accept[b][i]| <= 1e-3 for an evaluated test,
 * bit 31 set if the sampled token's CDF interval edge is within 1e-3 of its width from u*S.
 * q_dtype is the bs_dtype of q_logits.  All pointers dev.
 * Errors: BS_ESTATE (no verify step pending), BS_ESHAPE (B / k_max differ from the verify step),
 * BS_EINVAL (null, temperature < 0, bad q_dtype). */
bs_status bs_accept_resample(bs_ctx* ctx, int B, const int32_t* draft_tokens, const int32_t* draft_len,
                             int k_max, const void* q_logits /*NULL or [T_d,vocab]*/, int q_dtype,
                             float temperature, int eos_id, int emit_bonus,
                             const float* u_accept /*[B,k_max]*/, const float* u_sample /*[B]*/,
                             int32_t* n_accepted /*[B]*/, int32_t* out_tokens /*[B,k_max+1]*/,
                             int32_t* n_emitted /*[B]*/, uint32_t* near_tie /*[B]*/, void* stream);

/* Same rule applied to caller-supplied float32 logits [M, vocab] (dev, packed rows) instead of
 * the hidden rows of a verify step; needs no preceding bs_verify_step and any vocab >= 2 with
 * vocab <= the context's vocab.  Entry point for sampler-only tests (e.g. the chi-square check). */
bs_status bs_accept_resample_logits(bs_ctx* ctx, int B, int vocab, const float* logits,
                                    const int32_t* draft_tokens, const int32_t* draft_len, int k_max,
                                    const void* q_logits, int q_dtype, float temperature, int eos_id,
                                    int emit_bonus, const float* u_accept, const float* u_sample,
                                    int32_t* n_accepted, int32_t* out_tokens, int32_t* n_emitted,
                                    uint32_t* near_tie, void* stream);

/* For callers that cannot allocate or hold device memory for the library: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same rule, same arguments and same results as
 * bs_accept_resample_logits with the filter off, but with no context and no workspace: what the kernels keep between
 * launches (row packing, softmax statistics, sampling partials) lives in a 9 MiB device array built into the
 * library (one copy per GPU, held until the process ends).  The call allocates nothing and only enqueues kernels on
 * `stream` (the stream's device must be the current device).  Limits: B <= 1024, B * (k_max + 1) <= 2048 packed
 * rows, k_max <= BS_MAX_K, 2 <= vocab <= 262144; beyond them BS_ESHAPE.  A sequence whose draft_len or token ids are
 * out of range is skipped (n_accepted = n_emitted = 0, out_tokens = -1); there is no status word to poll.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams or host
 * threads) race; calls ordered on one stream do not.  Errors: BS_EINVAL (null, temperature < 0, bad q_dtype),
 * BS_ESHAPE, BS_EHIP (the array's address could not be obtained). */
bs_status bs_accept_resample_logits_noalloc(int B, int vocab, const float* logits, const int32_t* draft_tokens,
                                            const int32_t* draft_len, int k_max, const void* q_logits, int q_dtype,
                                            float temperature, int eos_id, int emit_bonus, const float* u_accept,
                                            const float* u_sample, int32_t* n_accepted, int32_t* out_tokens,
                                            int32_t* n_emitted, uint32_t* near_tie, void* stream);

/* Sec. 3.2 defines p_t as the decoding distribution "after temperature scaling and any top-p / top-k
 * filtering": selects that filtering for all following bs_accept_resample / bs_accept_resample_logits
 * calls of the context.  Tokens are ranked by logit (equal logits: lower index first); top_k keeps the
 * first top_k of the ranking (top_k <= 0 or >= vocab: off); top_p then keeps the shortest prefix of
 * what is left whose mass reaches top_p times the mass of what is left (top_p >= 1: off); the kept
 * probabilities are renormalised and take the place of p_i in the accept test, the residual and the
 * bonus / plain sample.  Temperature 0 is unaffected (the arg-max is always kept).
 * logits_scratch (dev, float32, at least B_max*(k_max+1)*vocab elements of the context's limits, owned
 * by the caller, must stay valid while the filter is on): bf16 models write every row's logits there,
 * because finding a row's threshold needs the row in memory (the unfiltered path keeps only per-tile
 * statistics); may be NULL for float32 models and for bs_accept_resample_logits.  Host call, no GPU
 * work.  Errors: BS_EINVAL (null ctx, top_p <= 0 or NaN); a filtered accept call fails with BS_ESTATE
 * if a bf16 model has no scratch and with BS_ESHAPE if vocab > 262136. */
bs_status bs_set_filter(bs_ctx* ctx, int top_k, float top_p, float* logits_scratch);

/* Alg. 1 "y <- y o a": keeps n_commit[b] of the k_b+1 tentative rows of the last verify step:
 * ctx_len[seq_slot[b]] += n_commit[b].  Normal use: n_commit = n_accepted + 1 (the last token and
 * the accepted drafts; the sampled token becomes the next step's last_token).  Prefill: verify a
 * chunk of prompt tokens as forced "drafts" and commit all k_b+1.  Rows beyond stay dead and are
 * overwritten by the next step (rollback).  n_commit dev [B].  Errors: BS_ESTATE, BS_ESHAPE,
 * BS_EINVAL; a value outside [0,k_b+1] sets BS_FAULT_COMMIT and leaves that slot unchanged. */
bs_status bs_kv_commit(bs_ctx* ctx, int B, const int32_t* seq_slot, const int32_t* n_commit,
                       void* stream);

/* Alg. 1 keeps the rollout y per sequence; its length on the cache side is the committed length c of the slot.
 * Copies ctx_len[seq_slot[b]] to ctx_len_out[b] for b < B (both dev), in stream order with the commits before
 * it.  (ctx_len itself is the caller's buffer and may also be read directly; this call gives the lengths of a
 * batch in batch order without the caller indexing by slot.)  A slot outside [0, n_slots) yields -1 and sets
 * BS_FAULT_SLOT.  Errors: BS_EINVAL (null), BS_ESHAPE (B < 1). */
bs_status bs_kv_lengths(bs_ctx* ctx, int B, const int32_t* seq_slot /*[B]*/, int32_t* ctx_len_out /*[B]*/, void* stream);

/* Cache import / export: copies n dense rows [n, Hkv, D] (dtype = desc.dtype, dev) of one layer
 * to / from positions pos0 .. pos0+n of a slot, through the block table.  Does not touch ctx_len.
 * Errors: BS_EINVAL, BS_ESHAPE (layer/slot out of range), BS_ECAPACITY (pos0+n beyond the slot). */
bs_status bs_kv_write(bs_ctx* ctx, int layer, int slot, int pos0, int n, const void* k_rows,
                      const void* v_rows, void* stream);
bs_status bs_kv_read(bs_ctx* ctx, int layer, int slot, int pos0, int n, void* k_rows, void* v_rows,
                     void* stream);

/* Measurement hooks (not part of Alg. 1): time every launch of one kernel class of the following
 * bs_verify_step / bs_accept_resample calls with HIP events recorded on the call's own stream.
 * bs_profile_begin selects the class (BS_PROF_*) and clears the counters; bs_profile_end synchronises
 * `stream` and returns the summed duration in milliseconds and the number of launches, then switches
 * the hooks off.  At most 4096 launches are timed per begin/end pair; later ones run untimed.
 * Errors: BS_EINVAL (null, unknown class), BS_EHIP. */
enum {
  BS_PROF_NONE = 0,
  BS_PROF_ATTENTION = 1,   /* ragged verify attention (bf16 models: the MFMA kernel, which also merges the token chunks) */
  BS_PROF_GEMM_QKV = 2,    /* QKV projection (bf16 models with head size 128: the kernel that also applies the
                              rotary embedding and appends K/V) */
  BS_PROF_GEMM_O = 3,
  BS_PROF_GEMM_GATE_UP = 4,
  BS_PROF_GEMM_DOWN = 5,
  BS_PROF_LMHEAD = 6,      /* LM-head GEMM with the softmax-statistics epilogue */
  BS_PROF_SAMPLE = 7,      /* residual / bonus inverse-CDF sampling */
  BS_PROF_LOOKUP = 8,      /* draft lookup */
  BS_PROF_EMPTY = 9        /* no kernel: one empty event pair per decoder layer of bs_verify_step, which measures
                              the fixed cost an event pair adds to every duration reported above */
};
bs_status bs_profile_begin(bs_ctx* ctx, int kernel_class);
bs_status bs_profile_end(bs_ctx* ctx, void* stream, float* total_ms /*host*/, int* launches /*host*/);

/* Synchronises `stream`, returns the device status word (BS_FAULT_* bits) and clears it. */
bs_status bs_poll_status(bs_ctx* ctx, void* stream, int32_t* fault_out /*host*/);

#ifdef __cplusplus
}
#endif
#endif /* BUBBLESPEC_H */
