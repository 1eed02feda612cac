// MoE routing: router logits come from the skinny GEMM (activations as one or two 16-bit terms, fp32
// accumulate, split-K planes); here: softmax top-k with renormalised weights,
// capture of the chosen expert ids (the record Rollout Routing Replay consumes,
// paper Sec. 5.5), and a stable, deterministic grouping of (token, slot) pairs by expert.
#include "kernels.h"

namespace rlx {
namespace {

constexpr int MAX_E = 256;

// Largest 64-bit key of the wave, returned to every lane.  Row-wise DPP steps (shifts by 1, 2, 4, 8 inside rows of
// 16 lanes, then the last lane of a row handed to the next row, then lane 31 to the upper half) leave the result
// in lane 63; a lane without a source at some step keeps its own key.  A chain of short-latency register moves
// instead of the six dependent cross-lane permutes of a butterfly, of which top-k would need eight in a row.
__device__ __forceinline__ unsigned long long wave_max_key(unsigned long long key) {
  uint32_t lo = (uint32_t)key, hi = (uint32_t)(key >> 32);
#define RLX_KEY_STEP(ctrl, row_mask)                                                           \
  {                                                                                            \
    const uint32_t olo = (uint32_t)__builtin_amdgcn_update_dpp((int)lo, (int)lo, ctrl, row_mask, 0xF, false); \
    const uint32_t ohi = (uint32_t)__builtin_amdgcn_update_dpp((int)hi, (int)hi, ctrl, row_mask, 0xF, false); \
    const bool take = ohi > hi || (ohi == hi && olo > lo);                                     \
    lo = take ? olo : lo;                                                                      \
    hi = take ? ohi : hi;                                                                      \
  }
  RLX_KEY_STEP(0x111, 0xF)   // row_shr:1
  RLX_KEY_STEP(0x112, 0xF)   // row_shr:2
  RLX_KEY_STEP(0x114, 0xF)   // row_shr:4
  RLX_KEY_STEP(0x118, 0xF)   // row_shr:8
  RLX_KEY_STEP(0x142, 0xA)   // row_bcast:15 into rows 1 and 3
  RLX_KEY_STEP(0x143, 0xC)   // row_bcast:31 into rows 2 and 3
#undef RLX_KEY_STEP
  const uint32_t rlo = (uint32_t)__builtin_amdgcn_readlane((int)lo, 63), rhi = (uint32_t)__builtin_amdgcn_readlane((int)hi, 63);
  return ((unsigned long long)rhi << 32) | rlo;
}
// floats as unsigned integers of the same order, and back
__device__ __forceinline__ uint32_t float_order_bits(float f) {
  const uint32_t u = __float_as_uint(f);
  return u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}
__device__ __forceinline__ float float_from_order_bits(uint32_t o) {
  return __uint_as_float(o ^ ((o >> 31) ? 0x80000000u : 0xFFFFFFFFu));
}

// Top-k of one token by one wave: lane holds experts lane, lane+64, ...; selection by (logit descending,
// id ascending); weights = softmax over the chosen logits (== softmax over all experts, renormalised).
__device__ __forceinline__ void wave_topk(const RouterArgs& a, int t, int lane, int32_t* idx_out, float* w_out) {
  // all plane loads go out first (the skips are uniform over the wave), then the sums in plane order
  constexpr int MAXP = 16;
  float v[MAX_E / 64];
  float part[MAX_E / 64][MAXP];
  const bool live = !a.tok_live || a.tok_live[t] != 0;   // requested with the logits, not after the selection
#pragma unroll
  for (int j = 0; j < MAX_E / 64; ++j) {
    const int e = lane + 64 * j;
    const int ec = e < a.E ? e : 0;
#pragma unroll
    for (int s = 0; s < MAXP; ++s)
      part[j][s] = (s < a.n_planes && 64 * j < a.E) ? a.logits[((size_t)s * a.T + t) * a.E + ec] : 0.f;
  }
#pragma unroll
  for (int j = 0; j < MAX_E / 64; ++j) {
    float acc = 0.f;
#pragma unroll
    for (int s = 0; s < MAXP; ++s) acc += s < a.n_planes ? part[j][s] : 0.f;
    v[j] = (lane + 64 * j) < a.E ? acc : -INFINITY;
  }
  float mx = -INFINITY;
#pragma unroll
  for (int j = 0; j < MAX_E / 64; ++j) mx = fmaxf(mx, v[j]);
  mx = wave_max(mx);
  float my_e = 0.f, denom = 0.f;
  int my_i = 0;
  const int32_t* replay = a.replay_idx ? a.replay_idx + ((size_t)t * a.n_layers + a.layer) * a.top_k : nullptr;
  for (int k = 0; k < a.top_k; ++k) {
    float bv = -INFINITY; int bi = 0x7FFFFFFF;
    bool given = false;                                        // uniform over the wave
    if (replay) {
      // routing replay (paper Sec. 5.5): the expert is given; its weight still comes from this layer's own gate
      // logits, renormalised over the replayed set.  An id outside [0, E), or one already taken by an earlier
      // slot of this token (its entry of v is -inf by then), is not used: the slot falls back to the layer's own
      // best expert not yet taken, so that a token never reaches an expert twice.
      bi = replay[k];
      if (bi >= 0 && bi < a.E) {
        float mine = -INFINITY;
#pragma unroll
        for (int j = 0; j < MAX_E / 64; ++j)
          if (j == (bi >> 6)) mine = v[j];
        bv = __shfl(mine, bi & 63, WAVE);
        given = bv != -INFINITY;
      }
    }
    if (!given) {
      bv = -INFINITY; bi = 0x7FFFFFFF;
#pragma unroll
      for (int j = 0; j < MAX_E / 64; ++j)
        if (v[j] > bv) { bv = v[j]; bi = lane + 64 * j; }      // ascending id within the lane
      // the wave's best by (logit descending, id ascending): the largest key (ordered logit bits, ~id)
      const unsigned long long best =
          wave_max_key(((unsigned long long)float_order_bits(bv) << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)bi));
      bv = float_from_order_bits((uint32_t)(best >> 32));
      bi = (int)(0xFFFFFFFFu - (uint32_t)best);
    }
    const float ev = __expf(bv - mx);
    denom += ev;
    if (lane == k) { my_e = ev; my_i = bi; }
    if ((bi & 63) == lane) {
#pragma unroll
      for (int j = 0; j < MAX_E / 64; ++j)
        if (j == (bi >> 6)) v[j] = -INFINITY;
    }
  }
  if (lane < a.top_k) {
    idx_out[lane] = my_i;
    w_out[lane] = my_e / denom;
    if (a.routing_out && live)
      a.routing_out[((size_t)t * a.n_layers + a.layer) * a.top_k + lane] = my_i;
  }
}

// grid = ceil(T / 4): every wave does the top-k of one token
__global__ __launch_bounds__(256) void moe_topk_kernel(RouterArgs a) {
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t < a.T) wave_topk(a, t, threadIdx.x & 63, a.topk_idx + (size_t)t * a.top_k, a.topk_w + (size_t)t * a.top_k);
}

// Stable counting sort of the T*top_k (token, slot) pairs by expert.  The pair list is cut into contiguous
// segments, one per wave.  Pass 1: per-segment histograms.  Scan: offsets by (expert, segment).  Pass 2: a pair's
// position = offset + its rank among equal experts, in pair order (the lanes holding the same expert are found
// with one ballot per id bit).  Short lists (decode) are sorted by one workgroup of four waves in one launch; long
// ones (prefill) by GROUP_WGS workgroups in three launches, the histograms and offsets passing through `seg_ws`.
constexpr int GROUP_WGS = 16;
constexpr int GROUP_SEGS = 4 * GROUP_WGS;
constexpr int GROUP_ONE_WG_PAIRS = 4096;

__device__ __forceinline__ int segment_len(int n_pairs, int n_segs) {   // a multiple of the wave size
  return ((n_pairs + n_segs - 1) / n_segs + 63) / 64 * 64;
}

__device__ __forceinline__ void count_segment(const int32_t* idx, int p_begin, int p_end, int E, int lane,
                                              int32_t* hist_w /*[MAX_E], LDS, zeroed*/) {
  for (int p0 = p_begin; p0 < p_end; p0 += 64) {
    const int p = p0 + lane;
    if (p < p_end) {
      const int e = idx[p];
      if (e >= 0 && e < E) atomicAdd(&hist_w[e], 1);
    }
  }
}

__device__ __forceinline__ void place_segment(const int32_t* idx, int p_begin, int p_end, int top_k, int E, int lane,
                                              int32_t* base_w /*[MAX_E], LDS: next free position per expert*/,
                                              int32_t* sorted_token, int32_t* pair_pos) {
  const unsigned long long lt = (1ull << lane) - 1ull;
  for (int p0 = p_begin; p0 < p_end; p0 += 64) {
    const int p = p0 + lane;
    const bool ok = p < p_end;
    int e = ok ? idx[p] : -1;
    if (e < 0 || e >= E) e = -1;
    unsigned long long same = __ballot(e >= 0);
#pragma unroll
    for (int bit = 0; bit < 8; ++bit) {
      const unsigned long long bal = __ballot((e >> bit) & 1);
      same &= ((e >> bit) & 1) ? bal : ~bal;
    }
    if (e >= 0) {
      const int b0 = base_w[e];
      const int pos = b0 + __popcll(same & lt);
      sorted_token[pos] = p / top_k;
      pair_pos[p] = pos;
      if ((same >> lane) >> 1 == 0) base_w[e] = b0 + __popcll(same);   // highest lane of the group
    }
  }
}

// one workgroup sorts the whole list
__global__ __launch_bounds__(256) void moe_group_kernel(RouterArgs a, int32_t* group_off, int32_t* sorted_token,
                                                        int32_t* pair_pos) {
  __shared__ int32_t hist[4 * MAX_E];
  __shared__ int32_t base[4 * MAX_E];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n_pairs = a.T * a.top_k, E = a.E;
  for (int i = threadIdx.x; i < 4 * MAX_E; i += 256) hist[i] = 0;
  __syncthreads();
  const int seg = segment_len(n_pairs, 4);
  const int p_begin = wave * seg, p_end = min(n_pairs, p_begin + seg);
  count_segment(a.topk_idx, p_begin, p_end, E, lane, hist + wave * MAX_E);
  __syncthreads();
  if (wave == 0) {   // exclusive scan over experts of the four-wave totals; lane holds experts 4*lane .. 4*lane+3
    int tot[4], run = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int e = 4 * lane + j;
      tot[j] = hist[e] + hist[MAX_E + e] + hist[2 * MAX_E + e] + hist[3 * MAX_E + e];
      run += tot[j];
    }
    int incl = run;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      int v = __shfl_up(incl, o, WAVE);
      if (lane >= o) incl += v;
    }
    int off = incl - run;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int e = 4 * lane + j;
      int b0 = off;
#pragma unroll
      for (int w = 0; w < 4; ++w) { base[w * MAX_E + e] = b0; b0 += hist[w * MAX_E + e]; }
      if (e < E) group_off[e] = off;
      off += tot[j];
    }
    if (lane == 63) group_off[E] = incl;
  }
  __syncthreads();
  place_segment(a.topk_idx, p_begin, p_end, a.top_k, E, lane, base + wave * MAX_E, sorted_token, pair_pos);
}

// long lists, launch 1 of 3 (grid GROUP_WGS): histogram of every segment -> seg_ws[segment][MAX_E]
__global__ __launch_bounds__(256) void moe_group_count_kernel(RouterArgs a, int32_t* seg_ws) {
  __shared__ int32_t hist[4 * MAX_E];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n_pairs = a.T * a.top_k;
  for (int i = threadIdx.x; i < 4 * MAX_E; i += 256) hist[i] = 0;
  __syncthreads();
  const int seg = segment_len(n_pairs, GROUP_SEGS), s = blockIdx.x * 4 + wave;
  const int p_begin = min(n_pairs, s * seg), p_end = min(n_pairs, p_begin + seg);
  count_segment(a.topk_idx, p_begin, p_end, a.E, lane, hist + wave * MAX_E);
  __syncthreads();
  for (int i = threadIdx.x; i < 4 * MAX_E; i += 256) seg_ws[(size_t)blockIdx.x * 4 * MAX_E + i] = hist[i];
}

// launch 2 of 3 (one workgroup, thread = expert): the counts of seg_ws become first positions, in place
// With tile_rows > 0 it also lists the row tiles of the grouped GEMMs that follow: item i = (expert, tile of
// tile_rows of its rows), experts ascending, then n_items .. max_items - 1 marked empty (-1).  A grid over
// (expert, tile index up to the longest expert could have) is mostly workgroups that find nothing to do; at 32 768
// tokens they were nine tenths of the grid and cost 3 % of the prefill.
__global__ __launch_bounds__(MAX_E) void moe_group_scan_kernel(int E, int32_t* seg_ws, int32_t* group_off, int tile_rows,
                                                               int max_items, int32_t* item_expert, int32_t* item_tile) {
  __shared__ int32_t tot[MAX_E];
  __shared__ int32_t tile0[MAX_E + 1];
  const int e = threadIdx.x;
  int32_t cnt[GROUP_SEGS];
#pragma unroll
  for (int s = 0; s < GROUP_SEGS; ++s) cnt[s] = seg_ws[(size_t)s * MAX_E + e];   // all loads go out together
  int run = 0;
#pragma unroll
  for (int s = 0; s < GROUP_SEGS; ++s) { const int c = cnt[s]; cnt[s] = run; run += c; }
  tot[e] = run;
  __syncthreads();
  const int my_tiles = (tile_rows > 0 && e < E) ? (run + tile_rows - 1) / tile_rows : 0;   // row tiles of expert e
  if (e < 64) {      // exclusive scans over experts (rows, row tiles), as in the one-workgroup kernel
    int t4[4], n4[4], sum = 0, nsum = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      t4[j] = tot[4 * e + j];
      sum += t4[j];
      n4[j] = (tile_rows > 0 && 4 * e + j < E) ? (t4[j] + tile_rows - 1) / tile_rows : 0;
      nsum += n4[j];
    }
    int incl = sum, nincl = nsum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int v = __shfl_up(incl, o, WAVE), nv = __shfl_up(nincl, o, WAVE);
      if (e >= o) { incl += v; nincl += nv; }
    }
    int off = incl - sum, noff = nincl - nsum;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      tot[4 * e + j] = off;
      tile0[4 * e + j] = noff;
      if (4 * e + j < E) group_off[4 * e + j] = off;
      off += t4[j];
      noff += n4[j];
    }
    if (e == 63) { group_off[E] = incl; tile0[MAX_E] = nincl; }
  }
  __syncthreads();
  if (tile_rows > 0) {
    for (int i = 0; i < my_tiles; ++i)
      if (tile0[e] + i < max_items) { item_expert[tile0[e] + i] = e; item_tile[tile0[e] + i] = i; }
    for (int i = tile0[MAX_E] + e; i < max_items; i += MAX_E) { item_expert[i] = -1; item_tile[i] = 0; }
  }
  const int off = tot[e];
#pragma unroll
  for (int s = 0; s < GROUP_SEGS; ++s) seg_ws[(size_t)s * MAX_E + e] = off + cnt[s];
}

// launch 3 of 3 (grid GROUP_WGS): every wave places the pairs of its segment
__global__ __launch_bounds__(256) void moe_group_place_kernel(RouterArgs a, const int32_t* seg_ws, int32_t* sorted_token,
                                                              int32_t* pair_pos) {
  __shared__ int32_t base[4 * MAX_E];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n_pairs = a.T * a.top_k;
  for (int i = threadIdx.x; i < 4 * MAX_E; i += 256) base[i] = seg_ws[(size_t)blockIdx.x * 4 * MAX_E + i];
  __syncthreads();
  const int seg = segment_len(n_pairs, GROUP_SEGS), s = blockIdx.x * 4 + wave;
  const int p_begin = min(n_pairs, s * seg), p_end = min(n_pairs, p_begin + seg);
  place_segment(a.topk_idx, p_begin, p_end, a.top_k, a.E, lane, base + wave * MAX_E, sorted_token, pair_pos);
}

}  // namespace

size_t moe_group_workspace_words() { return (size_t)GROUP_SEGS * MAX_E; }

bool moe_group_lists_items(int T, int top_k) { return (size_t)T * top_k > GROUP_ONE_WG_PAIRS; }

hipError_t moe_route(const RouterArgs& a, int32_t* group_off, int32_t* sorted_token, int32_t* pair_pos,
                     int32_t* seg_ws, bool group, int tile_rows, int max_items, int32_t* item_expert,
                     int32_t* item_tile, hipStream_t st) {
  hipLaunchKernelGGL(moe_topk_kernel, dim3((a.T + 3) / 4), dim3(256), 0, st, a);
  if (!group) return hipGetLastError();
  if ((size_t)a.T * a.top_k <= GROUP_ONE_WG_PAIRS) {
    hipLaunchKernelGGL(moe_group_kernel, dim3(1), dim3(256), 0, st, a, group_off, sorted_token, pair_pos);
  } else {
    hipLaunchKernelGGL(moe_group_count_kernel, dim3(GROUP_WGS), dim3(256), 0, st, a, seg_ws);
    hipLaunchKernelGGL(moe_group_scan_kernel, dim3(1), dim3(MAX_E), 0, st, a.E, seg_ws, group_off, tile_rows, max_items,
                       item_expert, item_tile);
    hipLaunchKernelGGL(moe_group_place_kernel, dim3(GROUP_WGS), dim3(256), 0, st, a, (const int32_t*)seg_ws,
                       sorted_token, pair_pos);
  }
  return hipGetLastError();
}

}  // namespace rlx
