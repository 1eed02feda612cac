/*
 * relax_rollout.h -- C ABI of the MI355X (gfx950) rollout-decode library.
 *
 * The library computes the rollout stage of the asynchronous RL engine of
 * arXiv 2604.11554 on one GPU: batched autoregressive decoding of a dense or MoE
 * decoder-only policy.  Per step it emits the fields that stage hands to the rest
 * of the system: the sampled token, its log-probability under the behaviour policy
 * (paper Sec. 3.3: responses and log probabilities are independent per-sample
 * fields; App. B.3: the trainer's importance ratios use them) and, for MoE
 * policies, the top-K expert indices taken at every MoE layer for every token, for
 * Rollout Routing Replay (paper Sec. 5.5).  Sequence state (a paged KV cache and
 * block table) persists across calls, so multi-turn sessions (paper Sec. 4.2) are
 * a sequence of prefill_chunk / decode_step calls.
 *
 * Conventions
 *  - Every array argument is a DEVICE pointer unless its comment says HOST.
 *  - All matrices are 16-bit floats (bf16, or IEEE fp16 for a model created with RLX_DTYPE_F16: the FP16
 *    precision option of the paper's FP16-vs-BF16 ablation) with logical shape [out_features, in_features]
 *    (y = x W^T).  One model uses one format for its weights, gains, embeddings and KV pages.
 *    The projection matrices and the LM head are passed in the library's packed
 *    streaming layout, produced from row-major storage by rlx_pack_weight; the
 *    embedding table and the norm gains stay row-major.
 *  - The caller owns every buffer (weights, KV pool, workspace, inputs, outputs);
 *    weights must outlive the model handle.  The library allocates device memory
 *    only in rlx_model_create (a few KB of pointer tables) and frees it in
 *    rlx_model_destroy; prefill/decode never allocate or synchronise.
 *  - `stream` is a hipStream_t passed as void*; calls only enqueue work on it.
 *    Results are valid once the caller has synchronised the stream.
 *  - Every function returns 0 on success or a negative RLX_E* code; nothing
 *    aborts, throws or prints.  rlx_last_error() gives a thread-local message.
 *    Arguments are validated on the host before the first launch: after an
 *    argument error (RLX_EINVAL, RLX_ENOMEM, RLX_EUNSUPPORTED) no work has been
 *    enqueued.  RLX_EHIP reports a failed launch part-way through a call: earlier
 *    launches of that call stay enqueued and its outputs are undefined.
 *  - Empty calls: a decode step with n_seqs == 0, and a chunk call (prefill, scoring)
 *    with n_seqs == 0 and total_tokens == 0, are valid: they return 0, enqueue nothing
 *    and read none of the arrays (which may be NULL).  A chunk call with sequences
 *    needs at least one token in all (total_tokens >= 1); single sequences of a chunk
 *    may be empty (cu_seqlens[i] == cu_seqlens[i+1]): nothing is appended or sampled for
 *    them and their outputs are pad / 0 / 0.  Negative counts are RLX_EINVAL.
 *  - A model handle is immutable after creation; concurrent calls must use
 *    distinct workspaces (and distinct sequences of the KV pool).
 */
#ifndef RELAX_ROLLOUT_H
#define RELAX_ROLLOUT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RLX_API __attribute__((visibility("default")))

#define RLX_OK 0
#define RLX_EINVAL (-1)       /* bad shape / NULL / limit exceeded                */
#define RLX_ENOMEM (-2)       /* workspace too small                              */
#define RLX_EHIP (-3)         /* a HIP runtime call failed                        */
#define RLX_EUNSUPPORTED (-4) /* shape outside what the kernels are built for     */

#define RLX_DTYPE_BF16 0
#define RLX_DTYPE_F16 1

typedef struct rlx_model rlx_model;

/* Shape of the policy.  Plain data, passed by const pointer. */
typedef struct {
  uint32_t struct_size;  /* = sizeof(rlx_model_config) */
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim; /* head_dim 64 or 128 */
  int32_t d_ff;                                               /* dense SwiGLU width, 0 for MoE */
  int32_t n_experts, top_k, d_ff_expert;                      /* 0,0,0 for dense; n_experts <= 256, top_k <= 8 */
  int32_t vocab;
  int32_t kv_block_size; /* tokens per KV page; must be 16 */
  float rms_eps;         /* RMSNorm epsilon, added to the mean square */
  float rope_theta;      /* rotary base; pair (i, i+head_dim/2) turns by pos*theta^(-2i/head_dim) */
  int32_t qk_norm;       /* 1: per-head RMSNorm of q and k before the rotary embedding */
  int32_t eos_token_id, pad_token_id;
  int32_t activation_split; /* 0: activations enter every matrix product as one 16-bit value (8 significand
                               bits for bf16, 11 for fp16);
                               1: as two bf16 terms (hi + lo, 16 significand bits; twice the MFMA work and
                               twice the activation traffic).  Must be 0 for RLX_DTYPE_F16: the low term of
                               an fp16 pair would mostly be subnormal (RLX_EUNSUPPORTED) */
  int32_t dtype;            /* RLX_DTYPE_BF16 or RLX_DTYPE_F16: format of every weight tensor, of input_embeds
                               and of the KV pool.  fp16 values past 65504 in magnitude (weights, keys, values or
                               activations entering a matrix product) become infinities: the caller picks fp16
                               only for models whose activations stay in range */
} rlx_model_config;

/*
 * Weights.  Scalars point at device tensors; the per-layer members are HOST arrays
 * of n_layers device pointers (copied at create).  Logical shapes (elements of the model's dtype); (P) marks
 * the tensors that must be in the packed layout (each expert matrix packed on its
 * own, experts stored back to back):
 *   embed [vocab, d_model]; lm_head (P) [vocab, d_model]; final_norm [d_model]
 *   attn_norm, ffn_norm [d_model]; q_norm, k_norm [head_dim] (NULL arrays if !qk_norm)
 *   wq (P) [n_q_heads*head_dim, d_model]; wk, wv (P) [n_kv_heads*head_dim, d_model]
 *   wo (P) [d_model, n_q_heads*head_dim]
 *   dense: w_gate_up (G) gate and up [d_ff, d_model] each; w_down (P) [d_model, d_ff]; w_router NULL
 *   MoE:   w_router (P) [n_experts, d_model]; w_gate_up (G) gate and up [n_experts, d_ff_expert, d_model] each;
 *          w_down (P) [n_experts, d_model, d_ff_expert]
 * (G): the gate and up matrices of a SwiGLU block interleaved into one packed [2 f, k]
 * matrix by rlx_pack_gate_up.
 * d_model, d_ff and d_ff_expert must be multiples of 16.  All pointers must be 16-byte aligned.
 */
typedef struct {
  uint32_t struct_size; /* = sizeof(rlx_weights) */
  const void* embed;
  const void* lm_head;
  const void* final_norm;
  const void* const* attn_norm;
  const void* const* wq;
  const void* const* wk;
  const void* const* wv;
  const void* const* wo;
  const void* const* q_norm;
  const void* const* k_norm;
  const void* const* ffn_norm;
  const void* const* w_gate_up;
  const void* const* w_down;
  const void* const* w_router;
} rlx_weights;

/*
 * Packed streaming layout of a [n, k] matrix (k a multiple of 16): rows are padded
 * to a multiple of 32 with zeros and stored as (n/32) x (k/16) blocks of 1 KB, block
 * (i, j) holding rows 32i..32i+31, columns 16j..16j+15 in the operand order of the
 * 32x32x16 MFMA on 16-bit operands (16-byte group g of a block = row 32i + g mod 32, columns
 * 16j + 8 (g div 32) .. +7), so that a wavefront streams a row tile as one contiguous
 * run.  rlx_pack_weight converts `count` row-major matrices stored back to back
 * (src, device) into `count` packed matrices stored back to back (dst, device, of
 * rlx_packed_weight_bytes(n, k) each).  src and dst must not overlap.
 */
RLX_API int rlx_packed_weight_bytes(int32_t n, int32_t k, size_t* bytes_out);
RLX_API int rlx_pack_weight(const void* src, void* dst, int32_t count, int32_t n, int32_t k, void* stream);
/*
 * Gate/up pair of a SwiGLU block: `count` row-major gate matrices [f, k] and up matrices
 * [f, k] (each set stored back to back) -> `count` packed [2 f, k] matrices whose 32-row
 * block row t holds gate rows 16t..16t+15 followed by up rows 16t..16t+15, so that one
 * wavefront produces both factors of silu(gate) * up for 16 features.  f %% 16 == 0.
 * Each output matrix takes rlx_packed_weight_bytes(2 f, k) bytes.
 */
RLX_API int rlx_pack_gate_up(const void* gate, const void* up, void* dst, int32_t count, int32_t f, int32_t k,
                             void* stream);

/* Create / destroy a model handle on the current HIP device. */
RLX_API int rlx_model_create(const rlx_model_config* cfg, const rlx_weights* w, rlx_model** out);
RLX_API int rlx_model_destroy(rlx_model* m);

/*
 * Tuning knob: the number of workgroups of the decode attention kernel.  A decode step lays the 32-key units of
 * all (sequence, KV head) pairs end to end and gives each workgroup a contiguous share (all within one unit of each other); the default is
 * two workgroups per compute unit (the grid that is exactly resident).  1 <= n_workgroups <= 1024; results do
 * not depend on it beyond the order in which partial softmax states are merged.  Not thread-safe against calls
 * that use the model.
 */
RLX_API int rlx_model_set_attention_grid(rlx_model* m, int32_t n_workgroups);

/*
 * Weight refresh between steps (the inference-engine end of the weight synchronisation of paper Sec. 3.2,
 * "Distributed Checkpoint Service", and the version v_r of the staleness rule s = v_t - v_r of Sec. 3.3,
 * "Unified training modes via staleness control").  rlx_model_set_weights replaces every weight pointer of the
 * model by those of `w` (same shapes, dtype and layouts as at create; the per-layer tables are copied) and
 * records `version`; nothing is copied on the device and no stream is touched.  Calls enqueued before it keep
 * reading the old tensors, calls made after it read the new ones, so:
 *   - the new tensors must be complete, on the stream of the next call or synchronised, before that call;
 *   - the old tensors may be released only once the calls enqueued before the swap have finished;
 *   - KV pages written under the old weights stay valid storage: a sequence that continues across the swap
 *     attends to keys and values of the old policy (a partial rollout), which is the caller's choice to allow.
 * On error (RLX_EINVAL: NULL or misaligned pointer, struct_size) the model keeps its previous weights and
 * version.  A model starts at version 0.  Not thread-safe against calls that use the model.
 * rlx_model_weight_version reports the version of the installed weights, i.e. the tag v_r of every token a
 * subsequent call emits.
 */
RLX_API int rlx_model_set_weights(rlx_model* m, const rlx_weights* w, uint64_t version);
RLX_API int rlx_model_weight_version(const rlx_model* m, uint64_t* version_out);

/*
 * The KV pool is the per-session state that persists across turns of a multi-turn rollout (paper Sec. 4.2,
 * "Custom rollout and reward": the rollout keeps session state between the model's turns and the tool outputs).
 * Size in bytes of a KV pool of n_blocks pages (2 bytes per element, the model's dtype).  Layout, private to the
 * library: [layer][block][kv_head]{ K[16][head_dim], V^T[head_dim][16] }.
 * The caller allocates it (256-byte aligned) and passes n_blocks to every call.
 */
RLX_API int rlx_kv_pool_bytes(const rlx_model* m, int64_t n_blocks, size_t* bytes_out);

/* Scratch bytes needed by calls with at most max_seqs sequences, max_tokens packed
 * tokens (a decode step has n_seqs tokens) and block-table rows of at most
 * max_blocks_per_seq entries.  256-byte aligned, caller-owned; holds no state
 * between calls. */
RLX_API int rlx_workspace_bytes(const rlx_model* m, int32_t max_seqs, int32_t max_tokens, int32_t max_blocks_per_seq,
                        size_t* bytes_out);

/* Copy whole KV pages src[i] -> dst[i] in every layer: copy-on-write of the partial tail page of a prompt that the
 * G responses of one sampling group share (paper Sec. 2.1, group-relative algorithms draw several responses per
 * prompt).  src/dst: device int32 [n]; pairs with an id outside [0, n_blocks) or src == dst are skipped. */
RLX_API int rlx_kv_copy_blocks(const rlx_model* m, void* kv_pool, int64_t n_blocks, const int32_t* src,
                       const int32_t* dst, int32_t n, void* stream);

/*
 * Block-table contract (both calls): block_table is int32 [n_seqs, max_blocks_per_seq];
 * entry j of a row is the physical page holding positions 16j..16j+15, in
 * [0, n_blocks).  Rows must cover every position the call reads or appends.  A
 * page may be listed by several sequences only while it is full and read-only;
 * a page receiving appends must belong to one sequence.
 *
 * Sampling contract: the token that will sit at absolute position p of a sequence
 * is argmax_v(z_v/T + g_v), g_v = -log(-log(u_v)), u_v = (R_v + 0.5) 2^-32, R_v =
 * word (v mod 4) of Philox-4x32-10 with key (seed lo, seed hi) and counter
 * (v div 4, p, 0, 0); ties go to the smaller v.  T <= 0 selects argmax_v z_v and
 * scores with T = 1.  The log-probability is log_softmax(z/T)[token].  A draw
 * depends only on (seed, position, v), never on the batch slot.
 *
 * Finish rule: with p the position of the emitted token, the token is replaced by
 * eos_token_id when p >= max_ctx_len - 1 (length cap); a sequence is finished once
 * it emits eos_token_id.  Finished rows are inert: no KV append, token =
 * pad_token_id, logprob = 0, routing rows untouched.
 */

/*
 * Prefill of one chunk: the generation stage's intake of prompt tokens, multimodal features and, between the turns
 * of an agentic rollout, tool outputs (paper Sec. 3.1, rollout produces the responses; Sec. 4.1, "Unified data
 * pipeline": placeholder positions are replaced by modality features; Sec. 4.2: tool results are appended to the
 * session).  The token it emits carries the per-sample fields of Sec. 3.3 ("field-based storage": response tokens
 * and log probabilities), and out_routing the expert indices that Sec. 5.5 records for every token.
 *
 * Append a chunk of known tokens to each of n_seqs sequences (varlen, packed) and,
 * where sample_last[i] != 0, emit the next token from the chunk's last position.
 * A sequence may contribute no token to a call (cu_seqlens[i] == cu_seqlens[i+1]); it then emits nothing.
 *   token_ids     int32 [total_tokens]; -1 = take the row of input_embeds instead
 *   input_embeds  [total_tokens, d_model] in the model's dtype, or NULL (rows used only where id == -1)
 *   cu_seqlens    int32 [n_seqs+1], cu_seqlens[0] = 0, cu_seqlens[n_seqs] = total_tokens
 *   ctx_lens      int32 [n_seqs] tokens already cached before this chunk (not modified)
 *   sample_last   uint8 [n_seqs]
 *   seeds uint64 [n_seqs]; temperature float [n_seqs]; max_ctx_len int32 [n_seqs]
 *   forced_tokens NULL or int32 [n_seqs] (teacher forcing; < 0 = not forced)
 *   out_tokens int32 [n_seqs]; out_logprobs float [n_seqs]; finished_out uint8 [n_seqs]
 *       (rows with sample_last == 0 get pad / 0 / 0)
 *   out_sampled   NULL or int32 [n_seqs]: the Gumbel-max draw before forcing / capping
 *   out_routing   NULL or int32 [total_tokens, n_layers, top_k] (MoE), descending gate probability
 *   out_logits    NULL or float [n_seqs, vocab] (debug; rows with sample_last == 0 hold the logits
 *                 of the chunk's last position as well)
 * total_tokens is a HOST integer equal to cu_seqlens[n_seqs].
 */
RLX_API int rollout_prefill_chunk(const rlx_model* m, void* kv_pool, int64_t n_blocks, void* workspace,
                          size_t workspace_bytes, int32_t n_seqs, int32_t total_tokens,
                          const int32_t* token_ids, const void* input_embeds, const int32_t* cu_seqlens,
                          const int32_t* ctx_lens, const int32_t* block_table, int32_t max_blocks_per_seq,
                          const uint8_t* sample_last, const uint64_t* seeds, const float* temperature,
                          const int32_t* max_ctx_len, const int32_t* forced_tokens, int32_t* out_tokens,
                          float* out_logprobs, uint8_t* finished_out, int32_t* out_sampled,
                          int32_t* out_routing, float* out_logits, void* stream);

/*
 * Teacher-forced scoring of a chunk with optional routing replay: the log-probability forward that consumes
 * what the rollout recorded (paper Sec. 3.3: per-token log-probabilities; Sec. 5.5: Rollout Routing Replay,
 * the experts chosen during generation are replayed in the later forward pass).  The chunk's tokens are
 * appended to the cache exactly as in rollout_prefill_chunk (so long sequences can be scored chunk by chunk);
 * nothing is sampled.  For every chunk position t with 0 <= target_ids[t] < vocab,
 *   out_logprobs[t] = log_softmax(z_t / T_i)[target_ids[t]],  z_t = logits after position t, i = its sequence;
 * other positions get 0.
 *   target_ids      int32 [total_tokens] (normally the next token of the same sequence; -1 = not scored)
 *   temperature     float [n_seqs] (<= 0 scores with T = 1)
 *   replay_routing  NULL or int32 [total_tokens, n_layers, top_k]: MoE layers use these experts instead of their
 *                   own top-k; the mixing weights are the layer's own gate probabilities renormalised over the
 *                   replayed set.  The K ids of a token must be distinct experts; an id outside
 *                   [0, n_experts), or one that repeats an earlier slot of the same token, is replaced by the
 *                   layer's own best expert not yet in the token's list (so no expert ever receives a token
 *                   twice).  Ignored for dense models.
 *   out_logprobs    float [total_tokens]
 *   out_routing     NULL or int32 [total_tokens, n_layers, top_k]: the experts used
 * token_ids, input_embeds, cu_seqlens, ctx_lens, block_table as in rollout_prefill_chunk.
 */
RLX_API int rollout_score_chunk(const rlx_model* m, void* kv_pool, int64_t n_blocks, void* workspace,
                        size_t workspace_bytes, int32_t n_seqs, int32_t total_tokens, const int32_t* token_ids,
                        const void* input_embeds, const int32_t* cu_seqlens, const int32_t* ctx_lens,
                        const int32_t* block_table, int32_t max_blocks_per_seq, const int32_t* target_ids,
                        const float* temperature, const int32_t* replay_routing, float* out_logprobs,
                        int32_t* out_routing, void* stream);

/*
 * The step the whole RL iteration waits on (paper Sec. 5.3: rollout generation is the longest stage of a step):
 * every live sequence emits one more response token with its log-probability (Sec. 3.3, per-sample fields) and,
 * for MoE policies, the experts chosen at every layer (Sec. 5.5, recorded "for every token during inference").
 *
 * One decode step for n_seqs sequences: each live row consumes tokens_inout[i] at
 * position ctx_lens_inout[i] (appending its K/V there) and emits the next token.
 *   tokens_inout    int32 [n_seqs]  in: last emitted token; out: new token (pad if finished)
 *   ctx_lens_inout  int32 [n_seqs]  in: cached length; out: +1 for rows live at entry
 *   finished_inout  uint8 [n_seqs]
 *   out_routing     NULL or int32 [n_seqs, n_layers, top_k]
 *   other arguments as in rollout_prefill_chunk.
 */
RLX_API int rollout_decode_step(const rlx_model* m, void* kv_pool, int64_t n_blocks, void* workspace,
                        size_t workspace_bytes, int32_t n_seqs, int32_t* tokens_inout,
                        int32_t* ctx_lens_inout, const int32_t* block_table, int32_t max_blocks_per_seq,
                        const uint64_t* seeds, const float* temperature, const int32_t* max_ctx_len,
                        uint8_t* finished_inout, const int32_t* forced_tokens, float* out_logprobs,
                        int32_t* out_sampled, int32_t* out_routing, float* out_logits, void* stream);

/*
 * rollout_decode_step for callers that cannot allocate device memory or keep a workspace of their own: code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation.  The step's scratch is a fixed array
 * of RLX_STATIC_WORKSPACE_BYTES that every GPU the library runs on holds from the moment the library's code is
 * loaded there until the process ends; the call allocates nothing, frees nothing and does not synchronise.
 * Arguments and results are those of rollout_decode_step without workspace / workspace_bytes; the model's device
 * must be the current device (as for every call).
 *   RLX_ENOMEM  the step needs more scratch than the array holds (rlx_workspace_bytes(m, n_seqs, n_seqs, ...) >
 *               RLX_STATIC_WORKSPACE_BYTES): nothing is enqueued; use rollout_decode_step with a workspace.
 * All calls on one GPU share that GPU's array: two calls of this entry point whose work overlaps in time on the
 * same GPU (different streams, or different threads) race on it and give undefined results; calls on one stream
 * are ordered and safe.  The array keeps the previous call's contents; no call depends on them.
 */
#define RLX_STATIC_WORKSPACE_BYTES (128u << 20)
RLX_API int rollout_decode_step_static(const rlx_model* m, void* kv_pool, int64_t n_blocks, int32_t n_seqs,
                        int32_t* tokens_inout, int32_t* ctx_lens_inout, const int32_t* block_table,
                        int32_t max_blocks_per_seq, const uint64_t* seeds, const float* temperature,
                        const int32_t* max_ctx_len, uint8_t* finished_inout, const int32_t* forced_tokens,
                        float* out_logprobs, int32_t* out_sampled, int32_t* out_routing, float* out_logits,
                        void* stream);

/*
 * Decode over shared prompt prefixes.  Sequences of one sampling group (the G responses drawn for one prompt by
 * the group-relative algorithms of paper Sec. 2.1, e.g. 8 per prompt) list the same physical pages for their
 * prompt in their block-table rows.  rollout_decode_step reads those pages once per sequence; with a descriptor
 * of the sharing, rollout_decode_step_shared reads them once per subgroup of 32 / (n_q_heads / n_kv_heads)
 * sequences, at most 16 (their query heads fill the matrix-core columns that one sequence leaves mostly empty:
 * two column tiles of 16) and merges
 * the two parts of each sequence's softmax.  The results equal rollout_decode_step's up to the order of the
 * floating-point merges.
 *
 *   rlx_shared_prefix_bytes   size of a descriptor for n_seqs sequences (device memory, caller-owned, 256-byte
 *                             aligned).
 *   rlx_shared_prefix_build   leader[i] (HOST int32 [n_seqs]) = first sequence of i's group (leader[i] <= i, a
 *                             group is a run of consecutive rows with one leader; leader[i] == i for a sequence on
 *                             its own); shared_pages[i] (HOST int32 [n_seqs]) = leading block-table entries of row
 *                             i that are identical to its leader's and hold full pages (16 cached tokens each).
 *                             The group shares min_i shared_pages[i] pages, rounded down to an even number.
 *                             Writes the descriptor to `desc` and synchronises `stream`.  RLX_EINVAL for a leader
 *                             outside 0..i or a negative count, RLX_ENOMEM if desc_bytes is too small.
 *                             Build it again whenever rows are added, removed or moved; it does not change while
 *                             the sequences only grow.  The library cannot check the claim of identical pages:
 *                             a descriptor that overstates the sharing gives wrong results (never an access
 *                             outside the pool).
 *   rollout_decode_step_shared  as rollout_decode_step, plus shared_prefix: a descriptor built for exactly n_seqs
 *                             rows (any other is ignored), or NULL.
 */
RLX_API int rlx_shared_prefix_bytes(const rlx_model* m, int32_t n_seqs, size_t* bytes_out);
RLX_API int rlx_shared_prefix_build(const rlx_model* m, int32_t n_seqs, const int32_t* leader,
                                    const int32_t* shared_pages, void* desc, size_t desc_bytes, void* stream);
RLX_API int rollout_decode_step_shared(const rlx_model* m, void* kv_pool, int64_t n_blocks, void* workspace,
                        size_t workspace_bytes, int32_t n_seqs, int32_t* tokens_inout,
                        int32_t* ctx_lens_inout, const int32_t* block_table, int32_t max_blocks_per_seq,
                        const uint64_t* seeds, const float* temperature, const int32_t* max_ctx_len,
                        uint8_t* finished_inout, const int32_t* forced_tokens, float* out_logprobs,
                        int32_t* out_sampled, int32_t* out_routing, float* out_logits,
                        const void* shared_prefix, void* stream);

/*
 * Single operators, exported for per-kernel parity tests and profiling.
 *   rlx_op_linear: y[t, n] = sum_k x[t, k] W[n, k]; x bf16 [n_tokens, k] row-major, W bf16
 *   [n, k] PACKED, y float [n_tokens, n]; runs the same weight-streaming kernel the decode
 *   step uses.  workspace: at least 2*32*ceil(n_tokens/32)*k + 16*4*n_tokens*n + 1024 bytes.
 */
RLX_API int rlx_op_linear(const void* x, const void* w, float* y, int32_t n_tokens, int32_t n, int32_t k,
                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * Timing aid for benchmarks.  Kernel classes of one layer of a step: */
#define RLX_K_NORM 1        /* residual add + RMSNorm                         */
#define RLX_K_QKV 2         /* q|k|v projection                               */
#define RLX_K_ROPE 3        /* q/k norm + rotary embedding + KV append        */
#define RLX_K_ATTN 4        /* paged attention (decode: per-share partials)   */
#define RLX_K_ATTN_MERGE 5  /* decode: merge of pairs that straddle shares     */
#define RLX_K_OPROJ 6       /* output projection                              */
#define RLX_K_GATEUP 7      /* gate/up projection + SwiGLU (dense or grouped) */
#define RLX_K_DOWN 8        /* down projection (dense or grouped)             */
#define RLX_K_ROUTER 9      /* MoE router logits                              */
#define RLX_K_GROUP 10      /* MoE top-k + capture (+ grouping pass, if one runs) */
#define RLX_K_LMHEAD 11     /* LM head + log-sum-exp / Gumbel-max partials    */
#define RLX_K_ATTN_PREFIX 12 /* decode: attention over shared prompt prefixes   */
/*
 * From now on every stride-th launch of `kernel_class` is bracketed with
 * hipEventRecord(start_events[i]) / hipEventRecord(stop_events[i]) on the call's
 * stream, i = 0, 1, ... until n_events pairs are used.  The arrays are HOST arrays
 * of caller-created hipEvent_t (timing enabled) that must stay alive until the
 * facility is switched off.  kernel_class == 0 switches it off and returns the
 * number of pairs recorded.  Process-wide state, not thread-safe; a debugging and
 * measurement facility only.
 */
RLX_API int rlx_profile_kernel(int32_t kernel_class, void* const* start_events, void* const* stop_events,
                               int32_t n_events, int32_t stride);

/* Thread-local text of the last error on this thread ("" if none). */
RLX_API const char* rlx_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* RELAX_ROLLOUT_H */
