// Paged GQA attention over the bf16 KV pool (gfx950, MFMA bf16 16x16x32).
//
// Pool page of one (layer, block, kv head):  K[16 tokens][hd]  then  V^T[hd][16 tokens].
// The transposed V page makes both contractions read 8 or 16 contiguous bytes per lane:
//   S^T[token, col]  = K[token, :] . Q[col, :]          A = K page rows,  B = Q columns
//   O^T[d, col]     += V^T[d, tokens] . P[tokens, col]  A = V^T rows,     B = P (registers of S^T)
// A "column" is one (query position, query head).  Decode: the 16 columns of a tile
// are the query heads of one KV head at the single new position (group <= 16), so a
// KV page is read once for all heads of its group.  Prefill: a tile is 16 consecutive
// positions of one head, causal mask per column.  The softmax statistics of a column
// live in the lanes that hold that column, so rescaling is lane-local; the max over
// keys is reduced across the four 16-lane groups with two shuffles.
#include "kernels.h"

namespace rlx {
namespace {

__device__ __forceinline__ bf16x8 load_2x4(const bf16_t* p0, const bf16_t* p1) {
  u32x2 a = *reinterpret_cast<const u32x2*>(p0);
  u32x2 b = *reinterpret_cast<const u32x2*>(p1);
  u32x4 v = {a[0], a[1], b[0], b[1]};
  return __builtin_bit_cast(bf16x8, v);
}

template <int HD, int NCT>
struct WaveState {
  float m[NCT], l[NCT];
  f32x4 o[NCT][HD / 16];
};

// merge the state held in LDS (written by another wave) into this wave's registers
template <int HD, int NCT>
__device__ __forceinline__ void merge_from_lds(WaveState<HD, NCT>& st, const float* ml, const f32x4* ob, int lane) {
#pragma unroll
  for (int c = 0; c < NCT; ++c) {
    float mb = ml[(c * 2 + 0) * WAVE + lane], lb = ml[(c * 2 + 1) * WAVE + lane];
    float mn = fmaxf(st.m[c], mb);
    float aa = (st.m[c] == -INFINITY) ? 0.f : __expf(st.m[c] - mn);
    float ab = (mb == -INFINITY) ? 0.f : __expf(mb - mn);
    st.l[c] = st.l[c] * aa + lb * ab;
    st.m[c] = mn;
#pragma unroll
    for (int dt = 0; dt < HD / 16; ++dt) {
      f32x4 v = ob[(c * (HD / 16) + dt) * WAVE + lane];
      st.o[c][dt] = st.o[c][dt] * aa + v * ab;
    }
  }
}

template <int HD, int NCT>
__device__ __forceinline__ void store_to_lds(const WaveState<HD, NCT>& st, float* ml, f32x4* ob, int lane) {
#pragma unroll
  for (int c = 0; c < NCT; ++c) {
    ml[(c * 2 + 0) * WAVE + lane] = st.m[c];
    ml[(c * 2 + 1) * WAVE + lane] = st.l[c];
#pragma unroll
    for (int dt = 0; dt < HD / 16; ++dt) ob[(c * (HD / 16) + dt) * WAVE + lane] = st.o[c][dt];
  }
}

template <int HD, int NCT, bool DECODE, int PL>
__global__ __launch_bounds__(256) void attn_kernel(AttnArgs a) {
  constexpr int DT = HD / 16, KS = HD / 32;
  __shared__ f32x4 lds_o[2][NCT * DT * WAVE];
  __shared__ float lds_ml[2][NCT * 2 * WAVE];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c16 = lane & 15, g = lane >> 4;
  const int group = a.Hq / a.Hkv;

  int seq, kvh, key_begin, key_end, split = 0, hbase = 0, q0 = 0, nq = 1, ctx;
  if (DECODE) {
    seq = blockIdx.x / a.Hkv;
    kvh = blockIdx.x % a.Hkv;
    split = blockIdx.y;
    if (!a.tok_live[seq]) return;
    ctx = a.ctx_lens[seq];
    key_begin = split * ATTN_SPLIT_TOKENS;
    key_end = min(ctx + 1, key_begin + ATTN_SPLIT_TOKENS);
    if (key_begin >= key_end) return;
  } else {
    if ((int)blockIdx.x >= a.n_qtiles[0]) return;
    seq = a.qtile_seq[blockIdx.x];
    q0 = a.qtile_q0[blockIdx.x];
    const int passes = (group + NCT - 1) / NCT;
    kvh = blockIdx.y / passes;
    hbase = (blockIdx.y % passes) * NCT;
    ctx = a.ctx_lens[seq];
    nq = a.cu_seqlens[seq + 1] - a.cu_seqlens[seq];
    key_begin = 0;
    key_end = ctx + min(q0 + 16, nq);
  }

  // ---- query fragments and per-column limits ----
  bf16x8 qf[PL][NCT][KS];
  int pos_col[NCT];
  bool col_ok[NCT];
  int trow[NCT], head[NCT];
#pragma unroll
  for (int c = 0; c < NCT; ++c) {
    if (DECODE) {
      head[c] = kvh * group + c16;
      col_ok[c] = c16 < group;
      trow[c] = seq;
      pos_col[c] = ctx;
    } else {
      head[c] = kvh * group + hbase + c;
      col_ok[c] = (hbase + c < group) && (q0 + c16 < nq);
      trow[c] = a.cu_seqlens[seq] + q0 + c16;
      pos_col[c] = ctx + q0 + c16;
    }
#pragma unroll
    for (int p = 0; p < PL; ++p)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        qf[p][c][ks] = col_ok[c] ? load_bf16x8(a.q.p + p * a.q.plane + ((size_t)trow[c] * a.Hq + head[c]) * HD +
                                               32 * ks + 8 * g)
                                 : zero_bf16x8();
  }

  WaveState<HD, NCT> st;
#pragma unroll
  for (int c = 0; c < NCT; ++c) {
    st.m[c] = -INFINITY; st.l[c] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) st.o[c][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  const float scale = rsqrtf((float)HD);
  const int32_t* table = a.block_table + (size_t)seq * a.max_blocks;
  const int blk_begin = key_begin >> 4;
  const int blk_end = (key_end + 15) >> 4;           // exclusive
  const int n_pairs = (blk_end - blk_begin + 1) >> 1;
  const size_t page = (size_t)2 * 16 * HD;           // elements of one (block, kv head)

  for (int pi = wave; pi < n_pairs; pi += 4) {
    const int j0 = blk_begin + 2 * pi, j1 = j0 + 1;
    const bool has1 = j1 < blk_end;
    int64_t b0 = (j0 < a.max_blocks) ? table[j0] : -1;
    int64_t b1 = (has1 && j1 < a.max_blocks) ? table[j1] : -1;
    const bool ok0 = b0 >= 0 && b0 < a.n_blocks, ok1 = b1 >= 0 && b1 < a.n_blocks;
    if (!ok0) b0 = 0;                                  // keep the loads in bounds; scores are masked below
    if (!ok1) b1 = b0;
    const bf16_t* kp0 = a.pool_layer + ((size_t)b0 * a.Hkv + kvh) * page;
    const bf16_t* kp1 = a.pool_layer + ((size_t)b1 * a.Hkv + kvh) * page;
    const bf16_t* vp0 = kp0 + 16 * HD;
    const bf16_t* vp1 = kp1 + 16 * HD;

    f32x4 s0[NCT], s1[NCT];
#pragma unroll
    for (int c = 0; c < NCT; ++c) { s0[c] = f32x4{0.f, 0.f, 0.f, 0.f}; s1[c] = f32x4{0.f, 0.f, 0.f, 0.f}; }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      bf16x8 k0 = load_bf16x8(kp0 + c16 * HD + 32 * ks + 8 * g);
      bf16x8 k1 = load_bf16x8(kp1 + c16 * HD + 32 * ks + 8 * g);
#pragma unroll
      for (int c = 0; c < NCT; ++c)
#pragma unroll
        for (int p = PL - 1; p >= 0; --p) {
          s0[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k0, qf[p][c][ks], s0[c], 0, 0, 0);
          s1[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k1, qf[p][c][ks], s1[c], 0, 0, 0);
        }
    }
    // V^T fragments: rows d = 16 dt + c16, tokens 4g..4g+3 of each of the two pages
    bf16x8 vf[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
      vf[dt] = load_2x4(vp0 + (size_t)(16 * dt + c16) * 16 + 4 * g, vp1 + (size_t)(16 * dt + c16) * 16 + 4 * g);

    bf16x8 pf[PL][NCT];
#pragma unroll
    for (int c = 0; c < NCT; ++c) {
      float mx = -INFINITY;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        int key0 = j0 * 16 + 4 * g + v, key1 = j1 * 16 + 4 * g + v;
        bool vis0 = ok0 && key0 < key_end && key0 <= pos_col[c];
        bool vis1 = ok1 && key1 < key_end && key1 <= pos_col[c];
        s0[c][v] = vis0 ? s0[c][v] * scale : -INFINITY;
        s1[c][v] = vis1 ? s1[c][v] * scale : -INFINITY;
        mx = fmaxf(mx, fmaxf(s0[c][v], s1[c][v]));
      }
      mx = fmaxf(mx, __shfl_xor(mx, 16, WAVE));
      mx = fmaxf(mx, __shfl_xor(mx, 32, WAVE));
      const float mn = fmaxf(st.m[c], mx);
      const float alpha = (st.m[c] == -INFINITY) ? 0.f : __expf(st.m[c] - mn);
      float p0[4], p1[4], ps = 0.f;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        p0[v] = (s0[c][v] == -INFINITY) ? 0.f : __expf(s0[c][v] - mn);
        p1[v] = (s1[c][v] == -INFINITY) ? 0.f : __expf(s1[c][v] - mn);
        ps += p0[v] + p1[v];
      }
      st.l[c] = st.l[c] * alpha + ps;     // partial over this lane's keys; lane groups are summed at the end
      st.m[c] = mn;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) st.o[c][dt] *= alpha;
      bf16_t ph[8], pl[8];
#pragma unroll
      for (int v = 0; v < 4; ++v) { split_bf16(p0[v], ph[v], pl[v]); split_bf16(p1[v], ph[4 + v], pl[4 + v]); }
      u32x4 pk = {(uint32_t)ph[0] | ((uint32_t)ph[1] << 16), (uint32_t)ph[2] | ((uint32_t)ph[3] << 16),
                  (uint32_t)ph[4] | ((uint32_t)ph[5] << 16), (uint32_t)ph[6] | ((uint32_t)ph[7] << 16)};
      pf[0][c] = __builtin_bit_cast(bf16x8, pk);
      if (PL == 2) {
        u32x4 pk2 = {(uint32_t)pl[0] | ((uint32_t)pl[1] << 16), (uint32_t)pl[2] | ((uint32_t)pl[3] << 16),
                     (uint32_t)pl[4] | ((uint32_t)pl[5] << 16), (uint32_t)pl[6] | ((uint32_t)pl[7] << 16)};
        pf[PL - 1][c] = __builtin_bit_cast(bf16x8, pk2);
      }
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int c = 0; c < NCT; ++c)
#pragma unroll
        for (int p = PL - 1; p >= 0; --p)
          st.o[c][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[dt], pf[p][c], st.o[c][dt], 0, 0, 0);
  }

  // denominators: sum the four lane groups' partial sums of each column
#pragma unroll
  for (int c = 0; c < NCT; ++c) {
    st.l[c] += __shfl_xor(st.l[c], 16, WAVE);
    st.l[c] += __shfl_xor(st.l[c], 32, WAVE);
  }

  // ---- fixed-order tree merge of the four waves: (0<-2, 1<-3), then 0<-1 ----
  if (wave >= 2) store_to_lds<HD, NCT>(st, lds_ml[wave - 2], lds_o[wave - 2], lane);
  __syncthreads();
  if (wave < 2) merge_from_lds<HD, NCT>(st, lds_ml[wave], lds_o[wave], lane);
  __syncthreads();
  if (wave == 1) store_to_lds<HD, NCT>(st, lds_ml[0], lds_o[0], lane);
  __syncthreads();
  if (wave != 0) return;
  merge_from_lds<HD, NCT>(st, lds_ml[0], lds_o[0], lane);

  // lane holds column c16, rows d = 16 dt + 4 g + {0..3}
#pragma unroll
  for (int c = 0; c < NCT; ++c) {
    if (!col_ok[c]) continue;
    if (DECODE) {
      float* dst = a.part + (((size_t)seq * a.Hq + head[c]) * a.n_splits + split) * (HD + 2);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) *reinterpret_cast<f32x4*>(dst + 16 * dt + 4 * g) = st.o[c][dt];
      if (g == 0) { dst[HD] = st.m[c]; dst[HD + 1] = st.l[c]; }
    } else {
      const float inv = st.l[c] > 0.f ? 1.f / st.l[c] : 0.f;
      const int mtiles = a.o.mtiles();
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        f32x4 v = st.o[c][dt] * inv;
        bf16_t hi[4], lo[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) split_bf16(v[j], hi[j], lo[j]);
        const int col = head[c] * HD + 16 * dt + 4 * g;   // feature index of the output projection's K
        bf16_t* dst = a.o.p + frag_act_offset(trow[c], col & ~7, 0, mtiles, PL) + (col & 7);
        u32x2 p = {(uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16)};
        *reinterpret_cast<u32x2*>(dst) = p;
        if (PL == 2) {
          u32x2 p2 = {(uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16)};
          *reinterpret_cast<u32x2*>(dst + 512) = p2;
        }
      }
    }
  }
}

// merge the decode splits of one (sequence, head) in split order and write bf16
template <int HD>
__global__ void attn_merge_kernel(AttnArgs a) {
  const int seq = blockIdx.x, head = blockIdx.y;
  const int d = threadIdx.x;   // HD threads
  const int col = head * HD + d;
  bf16_t* dst = a.o.p + frag_act_offset(seq, col & ~7, 0, a.o.mtiles(), a.o.planes) + (col & 7);
  if (!a.tok_live[seq]) {
    dst[0] = 0;
    if (a.o.planes == 2) dst[512] = 0;
    return;
  }
  const int n_keys = a.ctx_lens[seq] + 1;
  const int ns = min(a.n_splits, (n_keys + ATTN_SPLIT_TOKENS - 1) / ATTN_SPLIT_TOKENS);
  const float* base = a.part + ((size_t)seq * a.Hq + head) * a.n_splits * (HD + 2);
  float m = -INFINITY, l = 0.f, o = 0.f;
  for (int s = 0; s < ns; ++s) {
    const float* p = base + (size_t)s * (HD + 2);
    float ms = p[HD], ls = p[HD + 1];
    if (ms == -INFINITY) continue;
    float mn = fmaxf(m, ms);
    float aa = (m == -INFINITY) ? 0.f : __expf(m - mn);
    float ab = __expf(ms - mn);
    o = o * aa + p[d] * ab;
    l = l * aa + ls * ab;
    m = mn;
  }
  bf16_t hi, lo;
  split_bf16(l > 0.f ? o / l : 0.f, hi, lo);
  dst[0] = hi;
  if (a.o.planes == 2) dst[512] = lo;
}

}  // namespace

hipError_t attention_decode(const AttnArgs& a, hipStream_t st) {
  dim3 grid(a.n_seqs * a.Hkv, a.n_splits);
  const bool two = a.q.planes == 2;
  if (a.hd == 128) {
    if (two) hipLaunchKernelGGL((attn_kernel<128, 1, true, 2>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((attn_kernel<128, 1, true, 1>), grid, dim3(256), 0, st, a);
  } else {
    if (two) hipLaunchKernelGGL((attn_kernel<64, 1, true, 2>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((attn_kernel<64, 1, true, 1>), grid, dim3(256), 0, st, a);
  }
  return hipGetLastError();
}

hipError_t attention_decode_merge(const AttnArgs& a, hipStream_t st) {
  if (a.hd == 128) hipLaunchKernelGGL((attn_merge_kernel<128>), dim3(a.n_seqs, a.Hq), dim3(128), 0, st, a);
  else hipLaunchKernelGGL((attn_merge_kernel<64>), dim3(a.n_seqs, a.Hq), dim3(64), 0, st, a);
  return hipGetLastError();
}

hipError_t attention_prefill(const AttnArgs& a, hipStream_t st) {
  constexpr int NCT = 2;
  const int group = a.Hq / a.Hkv;
  const int passes = (group + NCT - 1) / NCT;
  dim3 grid(a.max_qtiles, a.Hkv * passes);
  const bool two = a.q.planes == 2;
  if (a.hd == 128) {
    if (two) hipLaunchKernelGGL((attn_kernel<128, NCT, false, 2>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((attn_kernel<128, NCT, false, 1>), grid, dim3(256), 0, st, a);
  } else {
    if (two) hipLaunchKernelGGL((attn_kernel<64, NCT, false, 2>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((attn_kernel<64, NCT, false, 1>), grid, dim3(256), 0, st, a);
  }
  return hipGetLastError();
}

}  // namespace rlx
