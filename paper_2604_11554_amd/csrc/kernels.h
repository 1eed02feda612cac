// Host-side launchers of the rollout kernels.  Every launcher only enqueues work on
// the given stream and returns hipGetLastError(); shapes are validated by the caller.
#pragma once
#include "common.h"

namespace rlx {

// Up to three row segments stacked into one logical [N, K] weight (q|k|v).
struct LinearW {
  const h16_t* seg[3];
  int rows[3];
  int N, K;
};
inline LinearW linear1(const void* w, int N, int K) {
  LinearW l = {};
  l.seg[0] = (const h16_t*)w; l.rows[0] = N; l.N = N; l.K = K;
  return l;
}

// A 16-bit activation matrix [T, K] in MFMA fragment order (common.h), carried as the sum of
// `planes` (1 or 2) terms of format `dtype` (DT_BF16 / DT_F16); two bf16 terms keep 16 significand bits.
// Kernels are built for bf16 with one or two terms and for fp16 with one term (the second term of an fp16 pair
// would mostly fall below the smallest normal fp16 number, 6.1e-5, and carry little).
// ss (optional): the rows are RMS-normalised rows WITHOUT their common factor: row t still has to be multiplied by
// 1 / sqrt((ss[4t] + ss[4t+1]) + (ss[4t+2] + ss[4t+3])) / K + eps), the four entries being the sums of squares of
// the four quarters of the row before the gain.  The norm kernel of short calls writes rows in this form (four
// workgroups per row instead of one) and the GEMM that consumes them applies the factor to its outputs, which is the
// same product in another order.
struct Act {
  h16_t* p;
  int T, K, planes, dtype;
  float* ss;
  float eps;
  __host__ __device__ int mtiles() const { return (T + 31) / 32; }
};
constexpr int NORM_PARTS = 4;
inline Act make_act(h16_t* p, int T, int K, int planes, int dtype) {
  Act a = {p, T, K, planes, dtype, nullptr, 0.f};
  return a;
}
// Row-major variant [planes][T, ld] (queries of the attention kernel).
struct RowAct {
  h16_t* p;
  size_t plane;
  int ld, planes, dtype;
};

// ---- gemm.hip ----
int gemm_max_splits();
void gemm_set_units(int n_units);   // compute units of the device (sizes the choice of tile form)
// number of split-K planes for y[T <= 256, N] = x W^T on a device with n_units compute units; the activations come
// as `planes` terms of format `dtype`
int gemm_plan_splits(int N, int K, int T, int max_splits, int n_units, int planes, int dtype);
// planes (1 or 2) for a call of more than 256 tokens: 2 where halving K lets the 256 x 256 form fill the device twice
int gemm_plan_splits_long(int N, int T, int planes, int dtype, int n_units);
// y[split][t][n] (fp32, leading dimension ldy); weights packed (common.h), activations in fragment order
hipError_t gemm_store(const LinearW& w, const Act& x, int T, float* y, int ldy, int splits, hipStream_t st);
// act[t][f] = silu(x Wg^T) * (x Wu^T); w_gate_up is the interleaved packed pair (pack_gate_up)
hipError_t gemm_swiglu(const h16_t* w_gate_up, int F, int K, const Act& x, int T, const Act& act, hipStream_t st);
int lmhead_tiles(int vocab);
// LM head with fused per-tile log-sum-exp and Gumbel-max partials: part[t][tile][4]
// row_seq (optional): row t reads temperature[row_seq[t]]; draw = false skips the Gumbel-max draw (scoring)
hipError_t gemm_lmhead(const h16_t* w_lm, int V, int K, const Act& x, int T, float* logits, float* part,
                       const uint64_t* seeds, const float* temperature, const int32_t* sample_pos,
                       const int32_t* row_seq, bool draw, hipStream_t st);
// expert-grouped forms: rows [group_off[e], group_off[e+1]) belong to expert e = blockIdx.y; max_rows bounds the rows
// of one expert, expected_rows (pairs / experts) picks the token-tile height
// items (optional, large-batch form only: gemm_grouped_item_rows() > 0): the list of (expert, row tile) pairs from
// moe_route; the grid then runs over the list instead of over (expert, tile index up to max_rows)
struct GroupItems { const int32_t* expert; const int32_t* tile; int max_items; };
// rows per tile of the form the grouped GEMMs take for this call if it can run over an item list, else 0
int gemm_grouped_item_rows(int E, int F, int N, const Act& x, int n_pairs, int expected_rows);
hipError_t gemm_grouped_swiglu(const h16_t* w_gate_up, int E, int F, int K, const Act& x, const int32_t* x_rows,
                               const int32_t* group_off, int max_rows, int expected_rows, const Act& act,
                               const GroupItems* items, hipStream_t st);
hipError_t gemm_grouped_store(const h16_t* w, int E, int N, int K, const Act& x,
                              const int32_t* group_off, int max_rows, int expected_rows, float* y,
                              const GroupItems* items, hipStream_t st);

// routed form of the gate/up GEMM (decode batches, two-term bf16): the kernel finds its expert's (token, slot) pairs
// in the routing table route_idx[n_pairs] itself, so no grouping pass runs before it; it writes act in expert order
// and publishes group_off[E + 1] and pair_pos[n_pairs] of that order for gemm_grouped_store and the combine.
bool gemm_routed_form(int E, int F, const Act& x, int n_pairs, int expected_rows);
hipError_t gemm_routed_swiglu(const h16_t* w_gate_up, int E, int F, int K, const Act& x, const int32_t* route_idx,
                              int n_pairs, int top_k, int max_rows, const Act& act, int32_t* group_off,
                              int32_t* pair_pos, hipStream_t st);

// ---- elementwise.hip ----
struct TokenMeta {        // per packed token, built on the device at the start of a call
  int32_t* tok_seq;       // sequence slot of token t
  int32_t* tok_pos;       // absolute position of token t
  uint8_t* tok_live;      // 0: row is inert (finished); no KV append
  int32_t* sample_row;    // [n_seqs] packed index of the token whose hidden state is sampled from
  int32_t* sample_pos;    // [n_seqs] absolute position of the token to be drawn
  uint8_t* sample_on;     // [n_seqs] 1 if the row emits a token in this call
  int32_t* qtile_seq;     // prefill attention tiles: sequence, first query index
  int32_t* qtile_q0;
  int32_t* n_qtiles;      // [1]
  int32_t* tok_iota;      // prefill: [T] 0, 1, 2, ... (row lists of the per-token scoring pass)
  float2* rope_cs;        // [T][hd/2] (cos, sin) of the rotary angles of each token's position
};
hipError_t meta_decode(const TokenMeta& m, int n_seqs, const int32_t* ctx_lens, const uint8_t* finished,
                       const double* inv_freq, int head_dim, hipStream_t st);
hipError_t meta_prefill(const TokenMeta& m, int n_seqs, int total_tokens, const int32_t* cu_seqlens,
                        const int32_t* ctx_lens, const uint8_t* sample_last, const double* inv_freq, int head_dim,
                        hipStream_t st);
hipError_t embed_tokens(const h16_t* embed, int vocab, int d, const int32_t* tokens, const h16_t* input_embeds,
                        int T, float* h, int dtype, hipStream_t st);

struct NormArgs {
  float* h;                  // [T, d] residual stream, updated in place when something is added
  const h16_t* gain;        // [d], format x.dtype
  int d, T;                  // T = number of output rows
  int T_total;               // rows of h (stride of the split-K planes)
  float eps;
  const int32_t* rows;       // optional: output row r normalises (and updates) h[rows[r]] only
  // optional additive term: (a) split-K planes  add[s][t][d], s < n_planes
  const float* add;
  int n_planes;
  // (b) MoE combine: sum_k w[t,k] * y[pair_pos[t*K+k]][d]
  const float* moe_y;
  const int32_t* pair_pos;
  const float* topk_w;
  int top_k;
  Act x;                     // [planes][T, d] normalised output
  float* xf;                 // optional fp32 copy of the normalised output
};
hipError_t rmsnorm(const NormArgs& a, hipStream_t st);
bool rmsnorm_in_parts(int d);   // whether rows of d elements can be written in the form of Act::ss

struct RopeArgs {
  const float* qkv;          // [n_planes][T, (Hq+2Hkv)*hd] fp32 split-K planes, summed in plane order
  int n_planes;
  const h16_t* q_gain;      // [hd] or null
  const h16_t* k_gain;
  const float2* rope_cs;     // [T][hd/2] (cos, sin) of each token's position (meta_decode / meta_prefill)
  int T, Hq, Hkv, hd;
  float eps;
  const int32_t* tok_seq; const int32_t* tok_pos; const uint8_t* tok_live;
  const int32_t* block_table; int max_blocks;
  h16_t* pool_layer;        // this layer's pages, elements of format q_out.dtype (as are the gains)
  int64_t n_blocks;
  RowAct q_out;              // [planes][T, Hq*hd]
};
hipError_t qk_rope_append(const RopeArgs& a, hipStream_t st);
// row-major [N, K] 16-bit -> packed streaming layout (rows padded to 32 with zeros); K % 16 == 0
hipError_t pack_weight(const h16_t* src, h16_t* dst, int N, int K, hipStream_t st);
// row-major gate [F, K] and up [F, K] -> one packed [2F, K] matrix whose 32-row tile t holds gate rows
// 16t..16t+15 followed by up rows 16t..16t+15 (F % 16 == 0)
hipError_t pack_gate_up(const h16_t* gate, const h16_t* up, h16_t* dst, int F, int K, hipStream_t st);
// row-major [T, K] 16-bit -> single-plane fragment order
hipError_t pack_activation(const h16_t* src, h16_t* dst, int T, int K, hipStream_t st);
// y[i] = sum_s planes[s][i], s ascending
hipError_t sum_planes(const float* planes, int n_planes, size_t n, float* y, hipStream_t st);
hipError_t kv_copy_blocks(h16_t* pool, int64_t n_blocks, int n_layers, size_t block_elems, const int32_t* src,
                          const int32_t* dst, int n, hipStream_t st);

// ---- attention.hip (prefill), attention_decode.hip ----
constexpr int ATTN_QTILE = 64;   // query positions per prefill attention workgroup (a 16-position tile per wave)
struct AttnArgs {            // prefill
  RowAct q;                  // [planes][T, Hq*hd]
  const h16_t* pool_layer;
  int64_t n_blocks;
  int Hq, Hkv, hd;
  const int32_t* block_table; int max_blocks;
  const int32_t* ctx_lens;   // cached length before this call, per sequence
  const int32_t* cu_seqlens;
  const int32_t* qtile_seq; const int32_t* qtile_q0; const int32_t* n_qtiles;
  int max_qtiles;
  Act o;                     // [T, Hq*hd] in fragment order (input of the output projection)
};
hipError_t attention_prefill(const AttnArgs& a, hipStream_t st);

struct AttnDecodeArgs {      // one new token per sequence: row = sequence slot
  RowAct q;                  // [planes][n_seqs, Hq*hd] rotated queries
  const h16_t* pool_layer;  // this layer's pages (the new token's K and V already appended)
  int64_t n_blocks;
  int Hq, Hkv, hd;
  const int32_t* block_table; int max_blocks;
  const int32_t* ctx_lens;   // cached length before this call = position of the new token
  int n_seqs;
  // plan of the step (attention_decode_plan): 32-key units of all (sequence, KV head) pairs end to end
  const int32_t* unit_prefix;  // [n_seqs + 1] exclusive prefix of the per-sequence unit counts (0 for inert rows)
  const int32_t* wg_seq;       // [n_wgs] sequence in which workgroup w's share starts
  const int32_t* plan_hdr;     // [4] units per share of the first H workgroups, total units, units per share of the others, H
  int n_wgs;                   // grid size: shares of the unit sequence
  float* part;               // [n_wgs][2][Hq/Hkv][hd+4] partial (o, m, l) of a share's first / other straddling pair
  Act o;                     // [n_seqs, Hq*hd] in fragment order (input of the output projection)
  // shared prompt prefixes (optional): the first units of a sequence that shares them with others are attended
  // once per group by attention_decode_prefix; the kernels above then start at unit sp.start_unit[seq]
  const int32_t* shared;     // descriptor built by shared_prefix_build (device), or null
  float* seq_part;           // [n_seqs][Hkv][Hq/Hkv][hd+4] partial of a pair that one share covered but a prefix precedes
  float* pre_part;           // [shared_prefix_max_tiles][SP_COLS][hd+4] partials of the prefix tiles
  int n_prefix_wgs;          // grid of the prefix kernel
};
// Descriptor of the shared prefixes of a batch, int32 words (built on the host, read by the kernels):
//   [0] n_seqs it was built for, [1] n_tiles, [2] members per tile MS = min(16, SP_COLS / (Hq/Hkv)), [3..7] 0
//   per sequence (4 arrays of n_seqs): start_unit, tile0 (first tile of its subgroup), n_chunks, col0 (its first column)
//   per tile (arrays of max_tiles): row (sequence whose block-table row lists the pages), kvh, unit lo, unit hi,
//   then members [max_tiles][16] (-1 = none).  Tile of (subgroup, chunk c, kvh) = tile0 + c * Hkv + kvh.
constexpr int SP_HDR = 8;
constexpr int SP_MAX_CHUNKS = 4;
constexpr int SP_COLS = 32;          // columns of a prefix tile: two matrix-core column tiles of 16
__host__ __device__ inline int shared_prefix_members(int group) { return group > 0 && SP_COLS / group < 16 ? SP_COLS / group : 16; }
// a subgroup has at least two members wherever the groups have, and at most one more subgroup per group than
// members / 2: tiles = subgroups x chunks x Hkv fit with at least one chunk each
__host__ __device__ inline int shared_prefix_max_tiles(int n_seqs, int Hkv) { return n_seqs * Hkv; }
inline size_t shared_prefix_words(int n_seqs, int Hkv) {
  return (size_t)SP_HDR + 4 * (size_t)n_seqs + (size_t)shared_prefix_max_tiles(n_seqs, Hkv) * (4 + 16);
}
// fills `words` (shared_prefix_words entries) from per-sequence group leaders and shared page counts (host arrays)
void shared_prefix_build(int n_seqs, int Hq, int Hkv, const int32_t* leader, const int32_t* shared_pages, int32_t* words);
hipError_t attention_decode_plan(int n_seqs, const int32_t* ctx_lens, const uint8_t* tok_live, int Hkv, int n_wgs,
                                 const int32_t* shared, int32_t* unit_prefix, int32_t* wg_seq, int32_t* hdr,
                                 hipStream_t st);
hipError_t attention_decode_prefix(const AttnDecodeArgs& a, hipStream_t st);   // no-op without a descriptor
hipError_t attention_decode(const AttnDecodeArgs& a, hipStream_t st);
hipError_t attention_decode_merge(const AttnDecodeArgs& a, hipStream_t st);   // prefix parts, straddling pairs, inert rows

// ---- moe.hip ----
struct RouterArgs {
  const float* logits;       // [n_planes][T, E] router logits (split-K planes, summed in plane order)
  int n_planes;
  int T, E, top_k;
  int32_t* topk_idx;         // [T, top_k]
  float* topk_w;             // [T, top_k]
  int32_t* routing_out;      // optional [T, n_layers, top_k] (this layer's slice is written)
  int layer, n_layers;
  const uint8_t* tok_live;   // rows that are inert leave routing_out untouched
  const int32_t* replay_idx; // optional [T, n_layers, top_k]: use these experts instead of the layer's own top-k
};
// top-k + renormalised weights + routing capture (one launch), then the stable grouping of the T*top_k
// (token, slot) pairs by expert: one more launch of one workgroup for short lists, three launches of several
// workgroups for long ones, which pass through `seg_ws` (moe_group_workspace_words() int32 words)
size_t moe_group_workspace_words();
// group = false: only the top-k launch (the routed gate/up GEMM reads topk_idx itself and publishes the grouping).
// Long lists (moe_group_lists_items) with tile_rows > 0: item_expert / item_tile[max_items] receive the list of
// (expert, tile of tile_rows rows) pairs that have rows, experts ascending, the rest marked -1; max_items must be at
// least T * top_k / tile_rows + E.
bool moe_group_lists_items(int T, int top_k);
hipError_t moe_route(const RouterArgs& a, int32_t* group_off, int32_t* sorted_token, int32_t* pair_pos,
                     int32_t* seg_ws, bool group, int tile_rows, int max_items, int32_t* item_expert,
                     int32_t* item_tile, hipStream_t st);

// ---- sampling.hip ----
struct FinalizeArgs {
  int n_rows, n_tiles, vocab, d;
  const float* part;          // [n_rows][n_tiles][4]
  Act x;                      // [planes][n_rows, d] final-normalised hidden
  const h16_t* w_lm;         // [vocab, d] packed, format x.dtype
  const float* temperature; const int32_t* max_ctx_len; const int32_t* forced;
  const int32_t* sample_pos; const uint8_t* sample_on;
  int eos, pad;
  int32_t* out_tokens; float* out_logprobs; int32_t* out_sampled;
  uint8_t* finished;          // decode: in/out; prefill: out
  int32_t* ctx_lens;          // decode: incremented for rows live at entry; null for prefill
  int is_decode;
  // scoring form: row r scores token forced[r] (>= 0) with temperature[row_seq[r]] and writes only
  // out_logprobs[r] (0 where forced[r] < 0); no length cap, no state update
  int score;
  const int32_t* row_seq;
};
hipError_t sample_finalize(const FinalizeArgs& a, hipStream_t st);

}  // namespace rlx
