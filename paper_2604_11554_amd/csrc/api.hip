// C ABI of the rollout library: handle lifetime, argument validation, workspace
// carving and the launch sequence of one prefill chunk / decode step.
#include "../../include/relax_rollout.h"

#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <new>
#include <vector>

#include "kernels.h"

using namespace rlx;

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

#define RLX_HIP(expr)                                                                        \
  do {                                                                                       \
    hipError_t e_ = (expr);                                                                  \
    if (e_ != hipSuccess) return fail(RLX_EHIP, "%s: %s", #expr, hipGetErrorString(e_));     \
  } while (0)

// Optional timing aid: launches of one kernel class are bracketed with caller-owned events.
struct ProfState {
  int cls = 0;
  void* const* start = nullptr;
  void* const* stop = nullptr;
  int n = 0, used = 0, stride = 1, seen = 0;
};
ProfState g_prof;

#define RLX_LAUNCH(cls_, expr)                                                               \
  do {                                                                                       \
    bool p_ = false;                                                                         \
    if (g_prof.cls == (cls_) && g_prof.used < g_prof.n) p_ = (g_prof.seen++ % g_prof.stride) == 0; \
    if (p_) RLX_HIP(hipEventRecord((hipEvent_t)g_prof.start[g_prof.used], st));              \
    RLX_HIP(expr);                                                                           \
    if (p_) RLX_HIP(hipEventRecord((hipEvent_t)g_prof.stop[g_prof.used++], st));             \
  } while (0)

size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

// Fixed scratch for callers that cannot allocate (rollout_decode_step_static): one array per GPU, resident from
// the moment the library's code is loaded on that GPU until the process ends.  Host code never uses the array's
// name as an address: scratch_on_device() asks the runtime once per device, with that device current, where that
// device's copy lives, and every launch receives the pointer it returned.
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[RLX_STATIC_WORKSPACE_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES] = {};

// device `dev` must be the current device
hipError_t scratch_on_device(int dev, void** out) {
  *out = nullptr;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

struct rlx_model {
  rlx_model_config cfg;
  const h16_t *embed, *lm_head, *final_norm;
  std::vector<const h16_t*> attn_norm, wq, wk, wv, wo, q_norm, k_norm, ffn_norm, w_gate_up, w_down, w_router;
  double* inv_freq;   // device, [head_dim / 2]
  int device;
  int n_units;        // compute units of the device
  int attn_wgs;       // decode attention grid: two workgroups per compute unit
  uint64_t weight_version;   // tag of the installed weights (rlx_model_set_weights)
  void* static_ws;           // this device's fixed scratch array (rollout_decode_step_static)
};

namespace {

struct Workspace {
  TokenMeta meta;
  float* h;          // [T, d]
  h16_t* xb;        // [planes][T, d]; every 16-bit activation buffer below has `planes` copies
  float* router;     // [planes][T, E] router logits (MoE)
  float* qkv;        // [planes][T, qkv_dim]
  h16_t* q;         // [T, q_dim]
  h16_t* ob;        // [T, q_dim]
  float* attn_part;  // [attn_wgs][2][Hq/Hkv][hd+4] decode partials of straddling (sequence, KV head) pairs
  int32_t *attn_prefix, *attn_wg_seq, *attn_hdr;   // decode attention plan
  float* attn_seq_part;   // [S][Hkv][Hq/Hkv][hd+4] own part of a pair that prefix tiles precede
  float* attn_pre_part;   // [shared_prefix_max_tiles][SP_COLS][hd+4] parts of the shared-prefix tiles
  float* planes;     // split-K planes of the o / down projections
  h16_t* act;       // dense [T, F]; MoE [T*top_k, Fe]
  float* moe_y;      // [T*top_k, d]
  int32_t* topk_idx; float* topk_w;
  int32_t *group_ws, *group_off, *sorted_token, *pair_pos;
  float* x_ss;                        // [T][4] sums of squares of the row quarters (norm of short calls, Act::ss)
  int32_t *item_expert, *item_tile;   // (expert, row tile) list of the grouped GEMMs of long calls
  int max_items;
  h16_t* x_lm;      // [S, d]
  float* lm_part;    // [S][tiles][4]
  size_t bytes;
};

constexpr int SCORE_ROWS = 256;      // rows per LM-head pass of rollout_score_chunk
constexpr int ATTN_WGS_MAX = 1024;   // decode attention grid limit (plan arrays are sized for it)

int plane_rows(int T) { return T <= 256 ? gemm_max_splits() * T : T; }

// carve the workspace; with base == nullptr only the size is computed
Workspace carve(const rlx_model_config& c, char* base, int S, int T, int max_blocks) {
  Workspace w = {};
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char* p = base ? base + off : nullptr;
    off += align_up(bytes);
    return p;
  };
  const int qdim = c.n_q_heads * c.head_dim, kvdim = c.n_kv_heads * c.head_dim;
  const int qkv_dim = qdim + 2 * kvdim;
  const int QT = T / 16 + S + 1;
  w.meta.tok_seq = (int32_t*)take((size_t)T * 4);
  w.meta.tok_pos = (int32_t*)take((size_t)T * 4);
  w.meta.tok_live = (uint8_t*)take((size_t)T);
  w.meta.sample_row = (int32_t*)take((size_t)S * 4);
  w.meta.sample_pos = (int32_t*)take((size_t)S * 4);
  w.meta.sample_on = (uint8_t*)take((size_t)S);
  w.meta.qtile_seq = (int32_t*)take((size_t)QT * 4);
  w.meta.qtile_q0 = (int32_t*)take((size_t)QT * 4);
  w.meta.n_qtiles = (int32_t*)take(4);
  w.meta.tok_iota = (int32_t*)take((size_t)T * 4);
  w.meta.rope_cs = (float2*)take((size_t)T * (c.head_dim / 2) * sizeof(float2));
  w.h = (float*)take((size_t)T * c.d_model * 4);
  const int PL = c.activation_split ? 2 : 1;
  w.xb = (h16_t*)take(frag_act_elems(T, c.d_model, PL) * 2);
  w.x_ss = (float*)take((size_t)T * NORM_PARTS * 4);
  w.router = c.n_experts ? (float*)take((size_t)plane_rows(T) * c.n_experts * 4) : nullptr;
  w.qkv = (float*)take((size_t)plane_rows(T) * qkv_dim * 4);
  w.q = (h16_t*)take((size_t)PL * T * qdim * 2);
  w.ob = (h16_t*)take(frag_act_elems(T, qdim, PL) * 2);
  w.attn_part = (float*)take((size_t)ATTN_WGS_MAX * 2 * (c.n_q_heads / c.n_kv_heads) * (c.head_dim + 4) * 4);
  w.attn_prefix = (int32_t*)take((size_t)(S + 1) * 4);
  w.attn_wg_seq = (int32_t*)take((size_t)ATTN_WGS_MAX * 4);
  w.attn_hdr = (int32_t*)take(4 * 4);
  w.attn_seq_part = (float*)take((size_t)S * c.n_q_heads * (c.head_dim + 4) * 4);
  w.attn_pre_part = (float*)take((size_t)shared_prefix_max_tiles(S, c.n_kv_heads) * SP_COLS * (c.head_dim + 4) * 4);
  // o / down planes: up to 16 per token for short calls, two for long ones (gemm_plan_splits_long)
  w.planes = (float*)take((size_t)(T <= 256 ? plane_rows(T) : 2 * T) * c.d_model * 4);
  if (c.n_experts) {
    const size_t P = (size_t)T * c.top_k;
    w.act = (h16_t*)take(frag_act_elems((int)P, c.d_ff_expert, PL) * 2);
    w.moe_y = (float*)take(P * c.d_model * 4);
    w.topk_idx = (int32_t*)take(P * 4);
    w.topk_w = (float*)take(P * 4);
    w.group_ws = (int32_t*)take(moe_group_workspace_words() * 4);
    w.group_off = (int32_t*)take((size_t)(c.n_experts + 1) * 4);
    w.sorted_token = (int32_t*)take(P * 4);
    w.pair_pos = (int32_t*)take(P * 4);
    w.max_items = (int)(P / 256) + c.n_experts;       // tiles of 256 rows: at most one partial tile per expert
    w.item_expert = (int32_t*)take((size_t)w.max_items * 4);
    w.item_tile = (int32_t*)take((size_t)w.max_items * 4);
  } else {
    w.act = (h16_t*)take(frag_act_elems(T, c.d_ff, PL) * 2);
  }
  const int lm_rows = S > SCORE_ROWS ? S : SCORE_ROWS;   // sampled rows of a call, or one block of scored rows
  w.x_lm = (h16_t*)take(frag_act_elems(lm_rows, c.d_model, PL) * 2);
  w.lm_part = (float*)take((size_t)lm_rows * lmhead_tiles(c.vocab) * 4 * 4);
  w.bytes = off;
  return w;
}

size_t block_elems(const rlx_model_config& c) { return (size_t)c.n_kv_heads * 2 * 16 * c.head_dim; }

struct StepIO {
  int n_seqs, T;
  bool decode;
  const int32_t* tokens; const h16_t* input_embeds;
  const int32_t* cu_seqlens; const int32_t* ctx_lens;
  const int32_t* block_table; int max_blocks;
  const uint64_t* seeds; const float* temperature; const int32_t* max_ctx_len; const int32_t* forced;
  int32_t* out_tokens; float* out_logprobs; uint8_t* finished; int32_t* out_sampled;
  int32_t* out_routing; float* out_logits;
  int32_t* ctx_lens_rw;   // decode only
  // scoring (rollout_score_chunk): every chunk position is scored against score_targets, nothing is sampled
  bool score; const int32_t* score_targets; float* score_logprobs;
  const int32_t* replay_routing;   // optional [T, n_layers, top_k]
  const int32_t* shared_prefix;    // decode only, optional descriptor of shared prompt prefixes
};

int run_layers(const rlx_model* m, h16_t* pool, int64_t n_blocks, const Workspace& w, const StepIO& io,
               hipStream_t st) {
  const rlx_model_config& c = m->cfg;
  const int d = c.d_model, T = io.T;
  const int qdim = c.n_q_heads * c.head_dim, kvdim = c.n_kv_heads * c.head_dim, qkv_dim = qdim + 2 * kvdim;
  const bool small = T <= 256;
  const int PL = c.activation_split ? 2 : 1;
  const int FMT = c.dtype;
  Act xb = make_act(w.xb, T, d, PL, FMT);
  const Act ob = make_act(w.ob, T, qdim, PL, FMT);
  const RowAct qb = {w.q, (size_t)T * qdim, qdim, PL, FMT};

  RLX_HIP(embed_tokens(m->embed, c.vocab, d, io.tokens, io.input_embeds, T, w.h, FMT, st));

  // residual contribution produced by the previous sub-layer, folded into the next norm
  const float* pend_planes = nullptr; int pend_n = 0; bool pend_moe = false;
  // MoE decode batches: the gate/up GEMM reads the routing table itself and publishes the grouping (no grouping launch)
  const int rows_per_expert = c.n_experts ? (int)(((long long)T * c.top_k + c.n_experts - 1) / c.n_experts) : 0;
  const bool routed = c.n_experts && small && gemm_routed_form(c.n_experts, c.d_ff_expert, xb, T * c.top_k, rows_per_expert);
  // long calls: the grouped GEMMs run over the list of (expert, row tile) items that the grouping pass writes
  const int item_rows = (c.n_experts && !small && moe_group_lists_items(T, c.top_k))
                            ? gemm_grouped_item_rows(c.n_experts, c.d_ff_expert, d, xb, T * c.top_k, rows_per_expert) : 0;
  // short calls: the norm runs as four workgroups per row and leaves the row's common factor to the GEMMs that read
  // xb (q|k|v, gate/up, router); not for fp16 (unnormalised rows would strain its range) and not where the grouped
  // gate/up goes through a row list
  if (small && FMT == DT_BF16 && rmsnorm_in_parts(d) && (c.n_experts == 0 || routed)) { xb.ss = w.x_ss; xb.eps = c.rms_eps; }
  const GroupItems items = {w.item_expert, w.item_tile, w.max_items};
  const GroupItems* itp = item_rows == 256 ? &items : nullptr;
  auto norm = [&](const h16_t* gain, const int32_t* rows, int n_rows, const Act& x, float* xf) -> hipError_t {
    NormArgs a = {};
    a.h = w.h; a.gain = gain; a.d = d; a.T = n_rows; a.T_total = T; a.eps = c.rms_eps; a.rows = rows;
    a.add = pend_planes; a.n_planes = pend_n;
    if (pend_moe) { a.moe_y = w.moe_y; a.pair_pos = w.pair_pos; a.topk_w = w.topk_w; a.top_k = c.top_k; }
    a.x = x; a.xf = xf;
    pend_planes = nullptr; pend_n = 0; pend_moe = false;
    return rmsnorm(a, st);
  };

  for (int l = 0; l < c.n_layers; ++l) {
    RLX_LAUNCH(RLX_K_NORM, norm(m->attn_norm[l], nullptr, T, xb, nullptr));
    LinearW wqkv = {};
    wqkv.seg[0] = m->wq[l]; wqkv.rows[0] = qdim;
    wqkv.seg[1] = m->wk[l]; wqkv.rows[1] = kvdim;
    wqkv.seg[2] = m->wv[l]; wqkv.rows[2] = kvdim;
    wqkv.N = qkv_dim; wqkv.K = d;
    const int s_qkv = small ? gemm_plan_splits(qkv_dim, d, T, gemm_max_splits(), m->n_units, PL, FMT) : 1;
    RLX_LAUNCH(RLX_K_QKV, gemm_store(wqkv, xb, T, w.qkv, qkv_dim, s_qkv, st));

    h16_t* pool_layer = pool + (size_t)l * n_blocks * block_elems(c);
    RopeArgs r = {};
    r.qkv = w.qkv; r.n_planes = s_qkv;
    r.q_gain = c.qk_norm ? m->q_norm[l] : nullptr; r.k_gain = c.qk_norm ? m->k_norm[l] : nullptr;
    r.rope_cs = w.meta.rope_cs;
    r.T = T; r.Hq = c.n_q_heads; r.Hkv = c.n_kv_heads; r.hd = c.head_dim;
    r.eps = c.rms_eps; r.tok_seq = w.meta.tok_seq; r.tok_pos = w.meta.tok_pos; r.tok_live = w.meta.tok_live;
    r.block_table = io.block_table; r.max_blocks = io.max_blocks;
    r.pool_layer = pool_layer; r.n_blocks = n_blocks; r.q_out = qb;
    RLX_LAUNCH(RLX_K_ROPE, qk_rope_append(r, st));
    if (io.decode) {
      AttnDecodeArgs at = {};
      at.q = qb; at.pool_layer = pool_layer; at.n_blocks = n_blocks;
      at.Hq = c.n_q_heads; at.Hkv = c.n_kv_heads; at.hd = c.head_dim;
      at.block_table = io.block_table; at.max_blocks = io.max_blocks; at.ctx_lens = io.ctx_lens;
      at.n_seqs = io.n_seqs; at.unit_prefix = w.attn_prefix; at.wg_seq = w.attn_wg_seq; at.plan_hdr = w.attn_hdr;
      at.n_wgs = m->attn_wgs; at.part = w.attn_part; at.o = ob;
      at.shared = io.shared_prefix; at.seq_part = w.attn_seq_part; at.pre_part = w.attn_pre_part;
      at.n_prefix_wgs = 2 * m->n_units;
      RLX_LAUNCH(RLX_K_ATTN_PREFIX, attention_decode_prefix(at, st));
      RLX_LAUNCH(RLX_K_ATTN, attention_decode(at, st));
      RLX_LAUNCH(RLX_K_ATTN_MERGE, attention_decode_merge(at, st));
    } else {
      AttnArgs at = {};
      at.q = qb; at.pool_layer = pool_layer; at.n_blocks = n_blocks;
      at.Hq = c.n_q_heads; at.Hkv = c.n_kv_heads; at.hd = c.head_dim;
      at.block_table = io.block_table; at.max_blocks = io.max_blocks; at.ctx_lens = io.ctx_lens;
      at.cu_seqlens = io.cu_seqlens; at.qtile_seq = w.meta.qtile_seq; at.qtile_q0 = w.meta.qtile_q0;
      at.n_qtiles = w.meta.n_qtiles; at.max_qtiles = T / ATTN_QTILE + io.n_seqs + 1; at.o = ob;
      RLX_LAUNCH(RLX_K_ATTN, attention_prefill(at, st));
    }

    const int s_o = small ? gemm_plan_splits(d, qdim, T, gemm_max_splits(), m->n_units, PL, FMT)
                          : gemm_plan_splits_long(d, T, xb.planes, xb.dtype, m->n_units);
    RLX_LAUNCH(RLX_K_OPROJ, gemm_store(linear1(m->wo[l], d, qdim), ob, T, w.planes, d, s_o, st));
    pend_planes = w.planes; pend_n = s_o;

    RLX_LAUNCH(RLX_K_NORM, norm(m->ffn_norm[l], nullptr, T, xb, nullptr));
    if (c.n_experts == 0) {
      const Act act = make_act(w.act, T, c.d_ff, PL, FMT);
      RLX_LAUNCH(RLX_K_GATEUP, gemm_swiglu(m->w_gate_up[l], c.d_ff, d, xb, T, act, st));
      const int s_d = small ? gemm_plan_splits(d, c.d_ff, T, gemm_max_splits(), m->n_units, PL, FMT)
                            : gemm_plan_splits_long(d, T, xb.planes, xb.dtype, m->n_units);
      RLX_LAUNCH(RLX_K_DOWN, gemm_store(linear1(m->w_down[l], d, c.d_ff), act, T, w.planes, d, s_d, st));
      pend_planes = w.planes; pend_n = s_d;
    } else {
      const int s_r = small ? gemm_plan_splits(c.n_experts, d, T, gemm_max_splits(), m->n_units, PL, FMT) : 1;
      RLX_LAUNCH(RLX_K_ROUTER, gemm_store(linear1(m->w_router[l], c.n_experts, d), xb, T, w.router, c.n_experts, s_r, st));
      RouterArgs ra = {};
      ra.logits = w.router; ra.n_planes = s_r; ra.T = T; ra.E = c.n_experts; ra.top_k = c.top_k;
      ra.topk_idx = w.topk_idx; ra.topk_w = w.topk_w; ra.routing_out = io.out_routing; ra.layer = l;
      ra.n_layers = c.n_layers; ra.tok_live = w.meta.tok_live; ra.replay_idx = io.replay_routing;
      RLX_LAUNCH(RLX_K_GROUP, moe_route(ra, w.group_off, w.sorted_token, w.pair_pos, w.group_ws, !routed, itp ? item_rows : 0,
                                         w.max_items, w.item_expert, w.item_tile, st));
      const Act act = make_act(w.act, T * c.top_k, c.d_ff_expert, PL, FMT);
      if (routed)
        RLX_LAUNCH(RLX_K_GATEUP, gemm_routed_swiglu(m->w_gate_up[l], c.n_experts, c.d_ff_expert, d, xb, w.topk_idx,
                                                    T * c.top_k, c.top_k, T, act, w.group_off, w.pair_pos, st));
      else
        RLX_LAUNCH(RLX_K_GATEUP, gemm_grouped_swiglu(m->w_gate_up[l], c.n_experts, c.d_ff_expert, d, xb,
                                                     w.sorted_token, w.group_off, T, rows_per_expert, act, itp, st));
      RLX_LAUNCH(RLX_K_DOWN, gemm_grouped_store(m->w_down[l], c.n_experts, d, c.d_ff_expert, act, w.group_off, T,
                                                rows_per_expert, w.moe_y, itp, st));
      pend_moe = true;
    }
  }

  if (io.score) {
    // every position is scored: final norm + LM head (log-sum-exp partials only, no draw) + target logit, in
    // blocks of SCORE_ROWS rows; each block applies the residual still pending from the last sub-layer to its rows
    const float* pp = pend_planes; const int pn = pend_n; const bool pm = pend_moe;
    for (int r0 = 0; r0 < T; r0 += SCORE_ROWS) {
      const int n = T - r0 < SCORE_ROWS ? T - r0 : SCORE_ROWS;
      const Act x_lm = make_act(w.x_lm, n, d, PL, FMT);
      pend_planes = pp; pend_n = pn; pend_moe = pm;
      RLX_HIP(norm(m->final_norm, w.meta.tok_iota + r0, n, x_lm, nullptr));
      RLX_LAUNCH(RLX_K_LMHEAD, gemm_lmhead(m->lm_head, c.vocab, d, x_lm, n, nullptr, w.lm_part, nullptr, io.temperature,
                                           nullptr, w.meta.tok_seq + r0, false, st));
      FinalizeArgs f = {};
      f.n_rows = n; f.n_tiles = lmhead_tiles(c.vocab); f.vocab = c.vocab; f.d = d;
      f.part = w.lm_part; f.x = x_lm; f.w_lm = m->lm_head;
      f.temperature = io.temperature; f.forced = io.score_targets + r0; f.row_seq = w.meta.tok_seq + r0;
      f.eos = c.eos_token_id; f.pad = c.pad_token_id; f.out_logprobs = io.score_logprobs + r0; f.score = 1;
      RLX_HIP(sample_finalize(f, st));
    }
    return RLX_OK;
  }

  // final norm of the rows that emit a token, LM head with fused log-sum-exp / Gumbel-max partials
  const int S = io.n_seqs;
  const Act x_lm = make_act(w.x_lm, S, d, PL, FMT);
  RLX_HIP(norm(m->final_norm, w.meta.sample_row, S, x_lm, nullptr));
  RLX_LAUNCH(RLX_K_LMHEAD, gemm_lmhead(m->lm_head, c.vocab, d, x_lm, S, io.out_logits, w.lm_part, io.seeds,
                                       io.temperature, w.meta.sample_pos, nullptr, true, st));
  FinalizeArgs f = {};
  f.n_rows = S; f.n_tiles = lmhead_tiles(c.vocab); f.vocab = c.vocab; f.d = d;
  f.part = w.lm_part; f.x = x_lm; f.w_lm = m->lm_head;
  f.temperature = io.temperature; f.max_ctx_len = io.max_ctx_len; f.forced = io.forced;
  f.sample_pos = w.meta.sample_pos; f.sample_on = w.meta.sample_on;
  f.eos = c.eos_token_id; f.pad = c.pad_token_id;
  f.out_tokens = io.out_tokens; f.out_logprobs = io.out_logprobs; f.out_sampled = io.out_sampled;
  f.finished = io.finished; f.ctx_lens = io.ctx_lens_rw; f.is_decode = io.decode ? 1 : 0;
  RLX_HIP(sample_finalize(f, st));
  return RLX_OK;
}

int check_common(const rlx_model* m, const void* kv_pool, int64_t n_blocks, const void* workspace, int32_t n_seqs,
                 int32_t max_blocks_per_seq) {
  if (!m) return fail(RLX_EINVAL, "model is NULL");
  if (!kv_pool || n_blocks <= 0) return fail(RLX_EINVAL, "kv_pool is NULL or n_blocks <= 0");
  if (!workspace) return fail(RLX_EINVAL, "workspace is NULL");
  if (n_seqs < 0 || n_seqs > (1 << 16)) return fail(RLX_EINVAL, "n_seqs %d out of range", n_seqs);
  if (max_blocks_per_seq <= 0 || max_blocks_per_seq > (1 << 20))
    return fail(RLX_EINVAL, "max_blocks_per_seq %d out of range", max_blocks_per_seq);
  if (!aligned16(kv_pool) || !aligned16(workspace)) return fail(RLX_EINVAL, "kv_pool/workspace not 16-byte aligned");
  return RLX_OK;
}

// Checks a weight table against the model's shape and installs its pointers (all or nothing).
int install_weights(rlx_model* m, const rlx_weights* wt) {
  const rlx_model_config& c = m->cfg;
  const bool moe = c.n_experts > 0;
  if (wt->struct_size != sizeof(rlx_weights)) return fail(RLX_EINVAL, "rlx_weights.struct_size mismatch");
  if (!wt->embed || !wt->lm_head || !wt->final_norm) return fail(RLX_EINVAL, "NULL global weight");
  if (!aligned16(wt->embed) || !aligned16(wt->lm_head) || !aligned16(wt->final_norm))
    return fail(RLX_EINVAL, "weights must be 16-byte aligned");
  const void* const* req[] = {wt->attn_norm, wt->wq, wt->wk, wt->wv, wt->wo, wt->ffn_norm, wt->w_gate_up, wt->w_down};
  for (auto p : req)
    if (!p) return fail(RLX_EINVAL, "NULL per-layer weight table");
  if (c.qk_norm && (!wt->q_norm || !wt->k_norm)) return fail(RLX_EINVAL, "qk_norm set but q_norm/k_norm missing");
  if (moe && !wt->w_router) return fail(RLX_EINVAL, "MoE model without w_router");
  struct Table { std::vector<const h16_t*>* dst; const void* const* src; };
  std::vector<const h16_t*> t[11];
  const Table tables[11] = {
      {&m->attn_norm, wt->attn_norm}, {&m->wq, wt->wq}, {&m->wk, wt->wk}, {&m->wv, wt->wv}, {&m->wo, wt->wo},
      {&m->ffn_norm, wt->ffn_norm}, {&m->w_gate_up, wt->w_gate_up}, {&m->w_down, wt->w_down},
      {&m->q_norm, c.qk_norm ? wt->q_norm : nullptr}, {&m->k_norm, c.qk_norm ? wt->k_norm : nullptr},
      {&m->w_router, moe ? wt->w_router : nullptr}};
  for (int i = 0; i < 11; ++i) {
    t[i].assign(c.n_layers, nullptr);
    if (!tables[i].src) continue;
    for (int l = 0; l < c.n_layers; ++l) {
      if (!tables[i].src[l] || !aligned16(tables[i].src[l]))
        return fail(RLX_EINVAL, "a per-layer weight pointer is NULL or not 16-byte aligned");
      t[i][l] = (const h16_t*)tables[i].src[l];
    }
  }
  for (int i = 0; i < 11; ++i) tables[i].dst->swap(t[i]);
  m->embed = (const h16_t*)wt->embed; m->lm_head = (const h16_t*)wt->lm_head;
  m->final_norm = (const h16_t*)wt->final_norm;
  return RLX_OK;
}

}  // namespace

extern "C" {

const char* rlx_last_error(void) { return g_err; }

int rlx_model_create(const rlx_model_config* cfg, const rlx_weights* wt, rlx_model** out) {
  if (!cfg || !wt || !out) return fail(RLX_EINVAL, "NULL argument");
  *out = nullptr;
  if (cfg->struct_size != sizeof(rlx_model_config)) return fail(RLX_EINVAL, "rlx_model_config.struct_size mismatch");
  const rlx_model_config& c = *cfg;
  if (c.n_layers <= 0 || c.d_model <= 0 || c.n_q_heads <= 0 || c.n_kv_heads <= 0 || c.vocab <= 0)
    return fail(RLX_EINVAL, "non-positive dimension");
  if (c.head_dim != 64 && c.head_dim != 128) return fail(RLX_EUNSUPPORTED, "head_dim %d (64 or 128)", c.head_dim);
  if (c.kv_block_size != 16) return fail(RLX_EUNSUPPORTED, "kv_block_size %d (must be 16)", c.kv_block_size);
  if (c.n_q_heads % c.n_kv_heads) return fail(RLX_EINVAL, "n_q_heads not a multiple of n_kv_heads");
  if (c.n_q_heads / c.n_kv_heads > 16) return fail(RLX_EUNSUPPORTED, "GQA group > 16");
  if (c.d_model % 16) return fail(RLX_EUNSUPPORTED, "d_model must be a multiple of 16");
  const bool moe = c.n_experts > 0;
  if (moe) {
    if (c.n_experts > 256 || c.top_k <= 0 || c.top_k > 8 || c.top_k > c.n_experts || c.d_ff_expert <= 0)
      return fail(RLX_EUNSUPPORTED, "MoE limits: n_experts <= 256, 1 <= top_k <= min(8, n_experts)");
    if (c.d_ff_expert % 16 || c.d_ff) return fail(RLX_EINVAL, "MoE: d_ff_expert %% 16 == 0 and d_ff == 0 required");
  } else {
    if (c.d_ff <= 0 || c.d_ff % 16) return fail(RLX_EINVAL, "dense: d_ff must be a positive multiple of 16");
    if (c.top_k || c.d_ff_expert) return fail(RLX_EINVAL, "dense: top_k and d_ff_expert must be 0");
  }
  if (c.eos_token_id < 0 || c.eos_token_id >= c.vocab || c.pad_token_id < 0 || c.pad_token_id >= c.vocab)
    return fail(RLX_EINVAL, "eos/pad token id outside the vocabulary");
  if (!(c.rms_eps >= 0.f) || !(c.rope_theta > 0.f)) return fail(RLX_EINVAL, "rms_eps / rope_theta");
  if (c.activation_split != 0 && c.activation_split != 1) return fail(RLX_EINVAL, "activation_split must be 0 or 1");
  if (c.qk_norm != 0 && c.qk_norm != 1) return fail(RLX_EINVAL, "qk_norm must be 0 or 1");
  if (c.dtype != RLX_DTYPE_BF16 && c.dtype != RLX_DTYPE_F16) return fail(RLX_EINVAL, "dtype must be RLX_DTYPE_BF16 or RLX_DTYPE_F16");
  if (c.dtype == RLX_DTYPE_F16 && c.activation_split)
    return fail(RLX_EUNSUPPORTED, "fp16 models carry activations as one term: activation_split must be 0");

  rlx_model* m = new (std::nothrow) rlx_model();
  if (!m) return fail(RLX_ENOMEM, "host allocation failed");
  m->cfg = c;
  m->inv_freq = nullptr;
  m->static_ws = nullptr;
  m->weight_version = 0;
  const int rc = install_weights(m, wt);
  if (rc != RLX_OK) {
    delete m;
    return rc;
  }
  // rotary frequencies theta^(-2i/hd) in double
  std::vector<double> inv(c.head_dim / 2);
  for (int i = 0; i < c.head_dim / 2; ++i) inv[i] = pow((double)c.rope_theta, -2.0 * i / c.head_dim);
  hipError_t e = hipGetDevice(&m->device);
  int n_cu = 0;
  if (e == hipSuccess) e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, m->device);
  m->n_units = n_cu > 0 ? n_cu : 1;
  gemm_set_units(m->n_units);
  m->attn_wgs = 2 * n_cu < ATTN_WGS_MAX ? (2 * n_cu > 0 ? 2 * n_cu : 1) : ATTN_WGS_MAX;
  if (e == hipSuccess && scratch_on_device(m->device, &m->static_ws) != hipSuccess) {
    // checked, not fatal: the model works with caller workspaces; rollout_decode_step_static reports the missing array
    m->static_ws = nullptr;
    (void)hipGetLastError();
  }
  if (e == hipSuccess) e = hipMalloc((void**)&m->inv_freq, inv.size() * sizeof(double));
  if (e == hipSuccess) e = hipMemcpy(m->inv_freq, inv.data(), inv.size() * sizeof(double), hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    if (m->inv_freq) (void)hipFree(m->inv_freq);
    delete m;
    return fail(RLX_EHIP, "rlx_model_create: %s", hipGetErrorString(e));
  }
  *out = m;
  return RLX_OK;
}

int rlx_model_set_attention_grid(rlx_model* m, int32_t n_workgroups) {
  if (!m) return fail(RLX_EINVAL, "model is NULL");
  if (n_workgroups < 1 || n_workgroups > ATTN_WGS_MAX)
    return fail(RLX_EINVAL, "rlx_model_set_attention_grid: n_workgroups %d outside 1..%d", n_workgroups, ATTN_WGS_MAX);
  m->attn_wgs = n_workgroups;
  return RLX_OK;
}

int rlx_model_set_weights(rlx_model* m, const rlx_weights* w, uint64_t version) {
  if (!m || !w) return fail(RLX_EINVAL, "rlx_model_set_weights: NULL argument");
  const int rc = install_weights(m, w);
  if (rc == RLX_OK) m->weight_version = version;
  return rc;
}

int rlx_model_weight_version(const rlx_model* m, uint64_t* version_out) {
  if (!m || !version_out) return fail(RLX_EINVAL, "rlx_model_weight_version: NULL argument");
  *version_out = m->weight_version;
  return RLX_OK;
}

int rlx_model_destroy(rlx_model* m) {
  if (!m) return RLX_OK;
  hipError_t e = m->inv_freq ? hipFree(m->inv_freq) : hipSuccess;
  delete m;
  if (e != hipSuccess) return fail(RLX_EHIP, "hipFree: %s", hipGetErrorString(e));
  return RLX_OK;
}

int rlx_kv_pool_bytes(const rlx_model* m, int64_t n_blocks, size_t* bytes_out) {
  if (!m || !bytes_out || n_blocks <= 0) return fail(RLX_EINVAL, "bad argument");
  *bytes_out = (size_t)m->cfg.n_layers * (size_t)n_blocks * block_elems(m->cfg) * 2;
  return RLX_OK;
}

int rlx_workspace_bytes(const rlx_model* m, int32_t max_seqs, int32_t max_tokens, int32_t max_blocks_per_seq,
                        size_t* bytes_out) {
  if (!m || !bytes_out || max_seqs <= 0 || max_tokens < max_seqs || max_blocks_per_seq <= 0)
    return fail(RLX_EINVAL, "bad argument (need 0 < max_seqs <= max_tokens, max_blocks_per_seq > 0)");
  // calls with at most 256 tokens keep up to 16 split-K planes per token, longer ones a single plane: the
  // need is monotonic in the token count on either side of that switch, not across it
  size_t b = carve(m->cfg, nullptr, max_seqs, max_tokens, max_blocks_per_seq).bytes;
  if (max_tokens > 256) {
    const size_t b2 = carve(m->cfg, nullptr, max_seqs < 256 ? max_seqs : 256, 256, max_blocks_per_seq).bytes;
    if (b2 > b) b = b2;
  }
  *bytes_out = b;
  return RLX_OK;
}

int rlx_kv_copy_blocks(const rlx_model* m, void* kv_pool, int64_t n_blocks, const int32_t* src, const int32_t* dst,
                       int32_t n, void* stream) {
  if (!m || !kv_pool || n_blocks <= 0 || n < 0 || (n > 0 && (!src || !dst))) return fail(RLX_EINVAL, "bad argument");
  RLX_HIP(kv_copy_blocks((h16_t*)kv_pool, n_blocks, m->cfg.n_layers, block_elems(m->cfg), src, dst, n,
                         (hipStream_t)stream));
  return RLX_OK;
}

int rollout_prefill_chunk(const rlx_model* m, void* kv_pool, int64_t n_blocks, void* workspace, size_t workspace_bytes,
                          int32_t n_seqs, int32_t total_tokens, const int32_t* token_ids, const void* input_embeds,
                          const int32_t* cu_seqlens, const int32_t* ctx_lens, const int32_t* block_table,
                          int32_t max_blocks_per_seq, const uint8_t* sample_last, const uint64_t* seeds,
                          const float* temperature, const int32_t* max_ctx_len, const int32_t* forced_tokens,
                          int32_t* out_tokens, float* out_logprobs, uint8_t* finished_out, int32_t* out_sampled,
                          int32_t* out_routing, float* out_logits, void* stream) {
  int rc = check_common(m, kv_pool, n_blocks, workspace, n_seqs, max_blocks_per_seq);
  if (rc) return rc;
  if (n_seqs == 0 && total_tokens == 0) return RLX_OK;   // an empty call: nothing to enqueue, no array is read
  if (n_seqs == 0 || total_tokens <= 0 || total_tokens > (1 << 24))
    return fail(RLX_EINVAL, "total_tokens %d out of range for %d sequences", total_tokens, n_seqs);
  if (!token_ids || !cu_seqlens || !ctx_lens || !block_table || !sample_last || !seeds || !temperature ||
      !max_ctx_len || !out_tokens || !out_logprobs || !finished_out)
    return fail(RLX_EINVAL, "NULL array argument");
  if (input_embeds && !aligned16(input_embeds)) return fail(RLX_EINVAL, "input_embeds not 16-byte aligned");
  const int T = total_tokens > n_seqs ? total_tokens : n_seqs;
  Workspace w = carve(m->cfg, (char*)workspace, n_seqs, T, max_blocks_per_seq);
  if (w.bytes > workspace_bytes)
    return fail(RLX_ENOMEM, "workspace too small: need %zu bytes, have %zu", w.bytes, workspace_bytes);
  hipStream_t st = (hipStream_t)stream;
  RLX_HIP(meta_prefill(w.meta, n_seqs, total_tokens, cu_seqlens, ctx_lens, sample_last, m->inv_freq, m->cfg.head_dim, st));
  StepIO io = {};
  io.n_seqs = n_seqs; io.T = total_tokens; io.decode = false;
  io.tokens = token_ids; io.input_embeds = (const h16_t*)input_embeds; io.cu_seqlens = cu_seqlens;
  io.ctx_lens = ctx_lens; io.block_table = block_table; io.max_blocks = max_blocks_per_seq;
  io.seeds = seeds; io.temperature = temperature; io.max_ctx_len = max_ctx_len; io.forced = forced_tokens;
  io.out_tokens = out_tokens; io.out_logprobs = out_logprobs; io.finished = finished_out;
  io.out_sampled = out_sampled; io.out_routing = m->cfg.n_experts ? out_routing : nullptr; io.out_logits = out_logits;
  return run_layers(m, (h16_t*)kv_pool, n_blocks, w, io, st);
}

int rollout_score_chunk(const rlx_model* m, void* kv_pool, int64_t n_blocks, void* workspace, size_t workspace_bytes,
                        int32_t n_seqs, int32_t total_tokens, const int32_t* token_ids, const void* input_embeds,
                        const int32_t* cu_seqlens, const int32_t* ctx_lens, const int32_t* block_table,
                        int32_t max_blocks_per_seq, const int32_t* target_ids, const float* temperature,
                        const int32_t* replay_routing, float* out_logprobs, int32_t* out_routing, void* stream) {
  int rc = check_common(m, kv_pool, n_blocks, workspace, n_seqs, max_blocks_per_seq);
  if (rc) return rc;
  if (n_seqs == 0 && total_tokens == 0) return RLX_OK;   // an empty call: nothing to enqueue, no array is read
  if (n_seqs == 0 || total_tokens <= 0 || total_tokens > (1 << 24))
    return fail(RLX_EINVAL, "total_tokens %d out of range for %d sequences", total_tokens, n_seqs);
  if (!token_ids || !cu_seqlens || !ctx_lens || !block_table || !target_ids || !temperature || !out_logprobs)
    return fail(RLX_EINVAL, "NULL array argument");
  if (input_embeds && !aligned16(input_embeds)) return fail(RLX_EINVAL, "input_embeds not 16-byte aligned");
  const int T = total_tokens > n_seqs ? total_tokens : n_seqs;
  Workspace w = carve(m->cfg, (char*)workspace, n_seqs, T, max_blocks_per_seq);
  if (w.bytes > workspace_bytes)
    return fail(RLX_ENOMEM, "workspace too small: need %zu bytes, have %zu", w.bytes, workspace_bytes);
  hipStream_t st = (hipStream_t)stream;
  RLX_HIP(meta_prefill(w.meta, n_seqs, total_tokens, cu_seqlens, ctx_lens, nullptr, m->inv_freq, m->cfg.head_dim, st));
  StepIO io = {};
  io.n_seqs = n_seqs; io.T = total_tokens; io.decode = false;
  io.tokens = token_ids; io.input_embeds = (const h16_t*)input_embeds; io.cu_seqlens = cu_seqlens;
  io.ctx_lens = ctx_lens; io.block_table = block_table; io.max_blocks = max_blocks_per_seq;
  io.temperature = temperature;
  io.out_routing = m->cfg.n_experts ? out_routing : nullptr;
  io.score = true; io.score_targets = target_ids; io.score_logprobs = out_logprobs;
  io.replay_routing = m->cfg.n_experts ? replay_routing : nullptr;
  return run_layers(m, (h16_t*)kv_pool, n_blocks, w, io, st);
}

int rollout_decode_step_shared(const rlx_model* m, void* kv_pool, int64_t n_blocks, void* workspace,
                               size_t workspace_bytes, int32_t n_seqs, int32_t* tokens_inout, int32_t* ctx_lens_inout,
                               const int32_t* block_table, int32_t max_blocks_per_seq, const uint64_t* seeds,
                               const float* temperature, const int32_t* max_ctx_len, uint8_t* finished_inout,
                               const int32_t* forced_tokens, float* out_logprobs, int32_t* out_sampled,
                               int32_t* out_routing, float* out_logits, const void* shared_prefix, void* stream) {
  int rc = check_common(m, kv_pool, n_blocks, workspace, n_seqs, max_blocks_per_seq);
  if (rc) return rc;
  if (n_seqs == 0) return RLX_OK;                         // an empty step: nothing to enqueue, no array is read
  if (!tokens_inout || !ctx_lens_inout || !block_table || !seeds || !temperature || !max_ctx_len ||
      !finished_inout || !out_logprobs)
    return fail(RLX_EINVAL, "NULL array argument");
  if (shared_prefix && !aligned16(shared_prefix)) return fail(RLX_EINVAL, "shared_prefix must be 16-byte aligned");
  Workspace w = carve(m->cfg, (char*)workspace, n_seqs, n_seqs, max_blocks_per_seq);
  if (w.bytes > workspace_bytes)
    return fail(RLX_ENOMEM, "workspace too small: need %zu bytes, have %zu", w.bytes, workspace_bytes);
  hipStream_t st = (hipStream_t)stream;
  RLX_HIP(meta_decode(w.meta, n_seqs, ctx_lens_inout, finished_inout, m->inv_freq, m->cfg.head_dim, st));
  RLX_HIP(attention_decode_plan(n_seqs, ctx_lens_inout, w.meta.tok_live, m->cfg.n_kv_heads, m->attn_wgs,
                                (const int32_t*)shared_prefix, w.attn_prefix, w.attn_wg_seq, w.attn_hdr, st));
  StepIO io = {};
  io.n_seqs = n_seqs; io.T = n_seqs; io.decode = true;
  io.tokens = tokens_inout; io.ctx_lens = ctx_lens_inout; io.ctx_lens_rw = ctx_lens_inout;
  io.block_table = block_table; io.max_blocks = max_blocks_per_seq;
  io.seeds = seeds; io.temperature = temperature; io.max_ctx_len = max_ctx_len; io.forced = forced_tokens;
  io.out_tokens = tokens_inout; io.out_logprobs = out_logprobs; io.finished = finished_inout;
  io.out_sampled = out_sampled; io.out_routing = m->cfg.n_experts ? out_routing : nullptr; io.out_logits = out_logits;
  io.shared_prefix = (const int32_t*)shared_prefix;
  return run_layers(m, (h16_t*)kv_pool, n_blocks, w, io, st);
}

int rollout_decode_step(const rlx_model* m, void* kv_pool, int64_t n_blocks, void* workspace, size_t workspace_bytes,
                        int32_t n_seqs, int32_t* tokens_inout, int32_t* ctx_lens_inout, const int32_t* block_table,
                        int32_t max_blocks_per_seq, const uint64_t* seeds, const float* temperature,
                        const int32_t* max_ctx_len, uint8_t* finished_inout, const int32_t* forced_tokens,
                        float* out_logprobs, int32_t* out_sampled, int32_t* out_routing, float* out_logits,
                        void* stream) {
  return rollout_decode_step_shared(m, kv_pool, n_blocks, workspace, workspace_bytes, n_seqs, tokens_inout,
                                    ctx_lens_inout, block_table, max_blocks_per_seq, seeds, temperature, max_ctx_len,
                                    finished_inout, forced_tokens, out_logprobs, out_sampled, out_routing, out_logits,
                                    nullptr, stream);
}

int rollout_decode_step_static(const rlx_model* m, void* kv_pool, int64_t n_blocks, int32_t n_seqs,
                               int32_t* tokens_inout, int32_t* ctx_lens_inout, const int32_t* block_table,
                               int32_t max_blocks_per_seq, const uint64_t* seeds, const float* temperature,
                               const int32_t* max_ctx_len, uint8_t* finished_inout, const int32_t* forced_tokens,
                               float* out_logprobs, int32_t* out_sampled, int32_t* out_routing, float* out_logits,
                               void* stream) {
  if (!m) return fail(RLX_EINVAL, "model is NULL");
  if (n_seqs < 0 || n_seqs > (1 << 16)) return fail(RLX_EINVAL, "n_seqs %d out of range", n_seqs);
  if (max_blocks_per_seq <= 0 || max_blocks_per_seq > (1 << 20))
    return fail(RLX_EINVAL, "max_blocks_per_seq %d out of range", max_blocks_per_seq);
  const size_t need = n_seqs ? carve(m->cfg, nullptr, n_seqs, n_seqs, max_blocks_per_seq).bytes : 0;
  if (need > (size_t)RLX_STATIC_WORKSPACE_BYTES)
    return fail(RLX_ENOMEM, "rollout_decode_step_static: a step of %d sequences of this model needs %zu bytes of "
                "scratch, the fixed array holds %zu; use rollout_decode_step with a workspace of your own", n_seqs,
                need, (size_t)RLX_STATIC_WORKSPACE_BYTES);
  if (!m->static_ws) return fail(RLX_EHIP, "rollout_decode_step_static: the fixed scratch array has no address");
  return rollout_decode_step_shared(m, kv_pool, n_blocks, m->static_ws, (size_t)RLX_STATIC_WORKSPACE_BYTES, n_seqs,
                                    tokens_inout, ctx_lens_inout, block_table, max_blocks_per_seq, seeds, temperature,
                                    max_ctx_len, finished_inout, forced_tokens, out_logprobs, out_sampled, out_routing,
                                    out_logits, nullptr, stream);
}

int rlx_shared_prefix_bytes(const rlx_model* m, int32_t n_seqs, size_t* bytes_out) {
  if (!m || !bytes_out || n_seqs <= 0 || n_seqs > (1 << 16)) return fail(RLX_EINVAL, "rlx_shared_prefix_bytes: bad argument");
  *bytes_out = align_up(shared_prefix_words(n_seqs, m->cfg.n_kv_heads) * 4);
  return RLX_OK;
}

int rlx_shared_prefix_build(const rlx_model* m, int32_t n_seqs, const int32_t* leader, const int32_t* shared_pages,
                            void* desc, size_t desc_bytes, void* stream) {
  if (!m || !leader || !shared_pages || !desc || n_seqs <= 0 || n_seqs > (1 << 16))
    return fail(RLX_EINVAL, "rlx_shared_prefix_build: bad argument");
  if (!aligned16(desc)) return fail(RLX_EINVAL, "rlx_shared_prefix_build: desc must be 16-byte aligned");
  const size_t words = shared_prefix_words(n_seqs, m->cfg.n_kv_heads);
  if (desc_bytes < words * 4) return fail(RLX_ENOMEM, "rlx_shared_prefix_build: desc needs %zu bytes", words * 4);
  for (int i = 0; i < n_seqs; ++i)
    if (leader[i] < 0 || leader[i] > i || shared_pages[i] < 0)
      return fail(RLX_EINVAL, "rlx_shared_prefix_build: sequence %d: leader %d (0..%d) / shared_pages %d", i, leader[i],
                  i, shared_pages[i]);
  std::vector<int32_t> host(words);
  shared_prefix_build(n_seqs, m->cfg.n_q_heads, m->cfg.n_kv_heads, leader, shared_pages, host.data());
  hipStream_t st = (hipStream_t)stream;
  RLX_HIP(hipMemcpyAsync(desc, host.data(), words * 4, hipMemcpyHostToDevice, st));
  RLX_HIP(hipStreamSynchronize(st));      // the staging vector dies with this call
  return RLX_OK;
}

int rlx_profile_kernel(int32_t kernel_class, void* const* start_events, void* const* stop_events, int32_t n_events,
                       int32_t stride) {
  if (kernel_class == 0 || n_events <= 0) {
    int used = g_prof.used;
    g_prof = ProfState();
    return used;
  }
  if (!start_events || !stop_events || stride <= 0 || kernel_class < 0 || kernel_class > RLX_K_ATTN_PREFIX)
    return fail(RLX_EINVAL, "rlx_profile_kernel: bad argument");
  g_prof = ProfState();
  g_prof.cls = kernel_class; g_prof.start = start_events; g_prof.stop = stop_events; g_prof.n = n_events;
  g_prof.stride = stride;
  return 0;
}

int rlx_packed_weight_bytes(int32_t n, int32_t k, size_t* bytes_out) {
  if (!bytes_out || n <= 0 || k <= 0 || (k % 16)) return fail(RLX_EINVAL, "rlx_packed_weight_bytes: k %% 16 == 0 required");
  *bytes_out = packed_weight_elems(n, k) * 2;
  return RLX_OK;
}

int rlx_pack_weight(const void* src, void* dst, int32_t count, int32_t n, int32_t k, void* stream) {
  if (!src || !dst || count <= 0 || n <= 0 || k <= 0 || (k % 16))
    return fail(RLX_EINVAL, "rlx_pack_weight: bad argument (k %% 16 == 0 required)");
  if (!aligned16(src) || !aligned16(dst)) return fail(RLX_EINVAL, "rlx_pack_weight: 16-byte alignment");
  const size_t pe = packed_weight_elems(n, k);
  for (int i = 0; i < count; ++i)
    RLX_HIP(pack_weight((const h16_t*)src + (size_t)i * n * k, (h16_t*)dst + (size_t)i * pe, n, k,
                        (hipStream_t)stream));
  return RLX_OK;
}

int rlx_pack_gate_up(const void* gate, const void* up, void* dst, int32_t count, int32_t f, int32_t k, void* stream) {
  if (!gate || !up || !dst || count <= 0 || f <= 0 || k <= 0 || (k % 16) || (f % 16))
    return fail(RLX_EINVAL, "rlx_pack_gate_up: bad argument (f %% 16 == 0 and k %% 16 == 0 required)");
  if (!aligned16(gate) || !aligned16(up) || !aligned16(dst)) return fail(RLX_EINVAL, "rlx_pack_gate_up: 16-byte alignment");
  const size_t pe = packed_weight_elems(2 * f, k);
  for (int i = 0; i < count; ++i)
    RLX_HIP(pack_gate_up((const h16_t*)gate + (size_t)i * f * k, (const h16_t*)up + (size_t)i * f * k,
                         (h16_t*)dst + (size_t)i * pe, f, k, (hipStream_t)stream));
  return RLX_OK;
}

int rlx_op_linear(const void* x, const void* w, float* y, int32_t n_tokens, int32_t n, int32_t k, void* workspace,
                  size_t workspace_bytes, void* stream) {
  if (!x || !w || !y || n_tokens <= 0 || n <= 0 || k <= 0 || (k % 16) || (n % 4))
    return fail(RLX_EINVAL, "rlx_op_linear: bad argument (k %% 16 == 0, n %% 4 == 0 required)");
  if (!aligned16(x) || !aligned16(w) || !aligned16(y) || !workspace || !aligned16(workspace))
    return fail(RLX_EINVAL, "rlx_op_linear: NULL workspace or 16-byte alignment");
  int dev = 0, n_units = 0;
  RLX_HIP(hipGetDevice(&dev));
  RLX_HIP(hipDeviceGetAttribute(&n_units, hipDeviceAttributeMultiprocessorCount, dev));
  const int splits = n_tokens <= 256 ? gemm_plan_splits(n, k, n_tokens, gemm_max_splits(), n_units > 0 ? n_units : 1, 1, DT_BF16) : 1;
  hipStream_t st = (hipStream_t)stream;
  const size_t xb = align_up(frag_act_elems(n_tokens, k, 1) * 2);
  const size_t pb = splits > 1 ? align_up((size_t)splits * n_tokens * n * 4) : 0;
  if (workspace_bytes < xb + pb) return fail(RLX_ENOMEM, "rlx_op_linear: workspace needs %zu bytes", xb + pb);
  h16_t* xp = (h16_t*)workspace;
  float* planes = (float*)((char*)workspace + xb);
  RLX_HIP(pack_activation((const h16_t*)x, xp, n_tokens, k, st));
  const Act xa = make_act(xp, n_tokens, k, 1, DT_BF16);
  if (splits == 1) {
    RLX_HIP(gemm_store(linear1(w, n, k), xa, n_tokens, y, n, 1, st));
    return RLX_OK;
  }
  RLX_HIP(gemm_store(linear1(w, n, k), xa, n_tokens, planes, n, splits, st));
  RLX_HIP(sum_planes(planes, splits, (size_t)n_tokens * n, y, st));
  return RLX_OK;
}

}  // extern "C"
