// Small memory-bound kernels: per-call token metadata, embedding gather, fused
// (residual add / split-K reduce / MoE combine) + RMSNorm, fused per-head q/k
// RMSNorm + rotary embedding + paged KV append, KV page copy.
#include "kernels.h"
#include "rope.h"

namespace rlx {
namespace {

// grid = n sequences, 64 threads: thread 0 writes the row's metadata, lane i < hd/2 the rotary factors of the
// row's new position (the same for every layer, so they are computed once per step and not per layer)
__global__ void meta_decode_kernel(TokenMeta m, int n, const int32_t* ctx, const uint8_t* fin, const double* inv_freq,
                                   int half) {
  const int i = blockIdx.x;
  const int pos = ctx[i];
  for (int j = threadIdx.x; j < half; j += blockDim.x) {
    float c, s;
    rope_cos_sin(pos, inv_freq, true, j, c, s);
    m.rope_cs[(size_t)i * half + j] = float2{c, s};
  }
  if (threadIdx.x != 0) return;
  uint8_t live = fin[i] ? 0 : 1;
  m.tok_seq[i] = i;
  m.tok_pos[i] = pos;
  m.tok_live[i] = live;
  m.sample_row[i] = i;
  m.sample_pos[i] = pos + 1;
  m.sample_on[i] = live;
}

// one workgroup; sequences are walked in order so the tile list is deterministic
__global__ void meta_prefill_kernel(TokenMeta m, int n_seqs, int total, const int32_t* cu, const int32_t* ctx,
                                    const uint8_t* sample_last) {
  __shared__ int tile_base[1025];
  // per-token fields: binary search of the owning sequence
  for (int t = threadIdx.x; t < total; t += blockDim.x) {
    int lo = 0, hi = n_seqs - 1;
    while (lo < hi) {
      int mid = (lo + hi + 1) >> 1;
      if (cu[mid] <= t) lo = mid; else hi = mid - 1;
    }
    m.tok_seq[t] = lo;
    m.tok_pos[t] = ctx[lo] + (t - cu[lo]);
    m.tok_live[t] = 1;
    m.tok_iota[t] = t;
  }
  for (int i = threadIdx.x; i < n_seqs; i += blockDim.x) {
    int len = cu[i + 1] - cu[i];
    m.sample_row[i] = len > 0 ? cu[i + 1] - 1 : -1;   // -1: no row (the final norm writes zeros, nothing is emitted)
    m.sample_pos[i] = ctx[i] + len;
    m.sample_on[i] = (sample_last && sample_last[i] && len > 0) ? 1 : 0;
  }
  // query tiles of ATTN_QTILE positions, sequence by sequence (n_seqs <= 1024 per chunk of the scan)
  __syncthreads();
  int base = 0;
  for (int s0 = 0; s0 < n_seqs; s0 += 1024) {
    int cnt = min(1024, n_seqs - s0);
    if (threadIdx.x == 0) {
      int acc = base;
      for (int i = 0; i < cnt; ++i) {
        tile_base[i] = acc;
        acc += (cu[s0 + i + 1] - cu[s0 + i] + ATTN_QTILE - 1) / ATTN_QTILE;
      }
      tile_base[cnt] = acc;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < cnt; i += blockDim.x) {
      int nt = tile_base[i + 1] - tile_base[i];
      for (int j = 0; j < nt; ++j) {
        m.qtile_seq[tile_base[i] + j] = s0 + i;
        m.qtile_q0[tile_base[i] + j] = ATTN_QTILE * j;
      }
    }
    base = tile_base[cnt];
    __syncthreads();
  }
  if (threadIdx.x == 0) m.n_qtiles[0] = base;
}

// grid = ceil(T / 4), a wave per token: the rotary factors of every token's position, once per call and not per
// (layer, head); the positions come from meta_prefill_kernel
__global__ __launch_bounds__(256) void rope_table_kernel(TokenMeta m, int total, const double* inv_freq, int half) {
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= total) return;
  const int pos = m.tok_pos[t];
  for (int j = threadIdx.x & 63; j < half; j += 64) {
    float c, s;
    rope_cos_sin(pos, inv_freq, true, j, c, s);
    m.rope_cs[(size_t)t * half + j] = float2{c, s};
  }
}

__global__ void embed_kernel(const h16_t* embed, int vocab, int d, const int32_t* tokens, const h16_t* inj, float* h,
                             int dtype) {
  int t = blockIdx.x;
  int tok = tokens[t];
  const h16_t* src;
  if (tok >= 0 && tok < vocab) src = embed + (size_t)tok * d;
  else if (tok < 0 && inj) src = inj + (size_t)t * d;
  else src = nullptr;   // out-of-range id: zero row rather than a stray read
  for (int i = threadIdx.x; i < d; i += blockDim.x) h[(size_t)t * d + i] = src ? h16_to_f32(src[i], dtype) : 0.f;
}

__device__ __forceinline__ float block_sum_256(float v, float* sh) {
  v = wave_sum(v);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = sh[0] + sh[1] + sh[2] + sh[3];
  __syncthreads();
  return r;
}

// One workgroup per row.  Every thread owns up to NV float4 slices of the row and issues all of its
// loads (residual, PR split-K planes per round, or the top-k expert rows) before the first add, so the
// kernel costs about one memory round trip per round; the host picks NV and PR so that a row of up to
// 4096 elements stays in registers and its planes take one round (two at 16 planes of the longest rows).
// The normalised row goes out in MFMA fragment order.
template <int NV, int PR>
__global__ __launch_bounds__(256) void rmsnorm_kernel(NormArgs a) {
  __shared__ float sh[4];
  const int r = blockIdx.x;
  const int t = a.rows ? a.rows[r] : r;
  const int nv = a.d >> 2;
  if (t < 0) {
    // no source row (a sequence that brought no token to this call): the output row is zero and the residual
    // stream is left alone.  Uniform over the workgroup, before any barrier.
    for (int i = threadIdx.x; i < nv; i += 256) {
      const int k = 4 * i;
      h16_t* xo = a.x.p + frag_act_offset(r, k & ~7, 0, a.x.mtiles(), a.x.planes) + (k & 7);
      const u32x2 z = {0u, 0u};
      *reinterpret_cast<u32x2*>(xo) = z;
      if (a.x.planes == 2) *reinterpret_cast<u32x2*>(xo + 512) = z;
      if (a.xf) *reinterpret_cast<f32x4*>(a.xf + (size_t)r * a.d + 4 * i) = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    return;
  }
  float* hrow = a.h + (size_t)t * a.d;
  const bool adding = (a.add != nullptr) || (a.moe_y != nullptr);
  const int mtiles = a.x.mtiles();
  const bool single = nv <= 256 * NV;
  const int dt = a.x.dtype;
  f32x4 keep[NV];
  u32x2 gain_k[NV];                          // gains of the kept slices, loaded with the row (not after the reduction)
  float ss = 0.f;
  int pp[8];
  float pw[8];
  if (a.moe_y) {
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const bool ok = k < a.top_k;
      pp[k] = ok ? a.pair_pos[t * a.top_k + k] : 0;
      pw[k] = ok ? a.topk_w[t * a.top_k + k] : 0.f;
    }
  }
  for (int base = 0; base < nv; base += 256 * NV) {
    // loads are unconditional at clamped addresses (slices past the row end re-read the last slice
    // and are never stored), so they all go out before the first add
    f32x4 v[NV];
    int ic[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int i = base + threadIdx.x + 256 * j;
      ic[j] = i < nv ? i : nv - 1;
      v[j] = *reinterpret_cast<const f32x4*>(hrow + 4 * ic[j]);
      if (single) gain_k[j] = *reinterpret_cast<const u32x2*>(a.gain + 4 * ic[j]);
    }
    if (a.add) {
      for (int s0 = 0; s0 < a.n_planes; s0 += PR) {    // PR planes per round, added in plane order
        f32x4 p[PR][NV];
#pragma unroll
        for (int q = 0; q < PR; ++q) {
          const int sc = s0 + q < a.n_planes ? s0 + q : a.n_planes - 1;
#pragma unroll
          for (int j = 0; j < NV; ++j)
            p[q][j] = *reinterpret_cast<const f32x4*>(a.add + ((size_t)sc * a.T_total + t) * a.d + 4 * ic[j]);
        }
#pragma unroll
        for (int q = 0; q < PR; ++q)
          if (s0 + q < a.n_planes) {
#pragma unroll
            for (int j = 0; j < NV; ++j) v[j] += p[q][j];
          }
      }
    }
    if (a.moe_y) {
      f32x4 y[8][NV];
#pragma unroll
      for (int k = 0; k < 8; ++k)
#pragma unroll
        for (int j = 0; j < NV; ++j) y[k][j] = *reinterpret_cast<const f32x4*>(a.moe_y + (size_t)pp[k] * a.d + 4 * ic[j]);
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int k = 0; k < 8; ++k) acc += y[k][j] * pw[k];     // slot order k = 0..K-1; unused slots weigh 0
        v[j] += acc;
      }
    }
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int i = base + threadIdx.x + 256 * j;
      if (i < nv) {
        if (adding) *reinterpret_cast<f32x4*>(hrow + 4 * i) = v[j];
        ss += v[j][0] * v[j][0] + v[j][1] * v[j][1] + v[j][2] * v[j][2] + v[j][3] * v[j][3];
      }
      if (single) keep[j] = v[j];
    }
  }
  const float tot = block_sum_256(ss, sh);
  const float rstd = 1.0f / sqrtf(tot / (float)a.d + a.eps);
  for (int base = 0; base < nv; base += 256 * NV) {
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int i = base + threadIdx.x + 256 * j;
      if (i >= nv) continue;
      const f32x4 hv = single ? keep[j] : *reinterpret_cast<const f32x4*>(hrow + 4 * i);   // own writes
      const u32x2 gb = single ? gain_k[j] : *reinterpret_cast<const u32x2*>(a.gain + 4 * i);
      f32x4 o;
      o[0] = hv[0] * rstd * h16_to_f32((h16_t)(gb[0] & 0xFFFFu), dt);
      o[1] = hv[1] * rstd * h16_to_f32((h16_t)(gb[0] >> 16), dt);
      o[2] = hv[2] * rstd * h16_to_f32((h16_t)(gb[1] & 0xFFFFu), dt);
      o[3] = hv[3] * rstd * h16_to_f32((h16_t)(gb[1] >> 16), dt);
      h16_t hi[4], lo[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) split_h16(o[e], hi[e], lo[e], dt);
      const int k = 4 * i;
      h16_t* xo = a.x.p + frag_act_offset(r, k & ~7, 0, mtiles, a.x.planes) + (k & 7);
      u32x2 pk = {(uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16)};
      *reinterpret_cast<u32x2*>(xo) = pk;
      if (a.x.planes == 2) {
        u32x2 pk2 = {(uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16)};
        *reinterpret_cast<u32x2*>(xo + 512) = pk2;
      }
      if (a.xf) *reinterpret_cast<f32x4*>(a.xf + (size_t)r * a.d + 4 * i) = o;
    }
  }
}

// Short calls: NORM_PARTS workgroups per row, each a quarter of it.  The kernel above puts a whole row (its
// residual and up to sixteen planes, ~100 KB at the 4B shape) through one compute unit, which takes in ~40 GB/s:
// 2.3 us of its 7-8.  A quarter of a row cannot know the row's sum of squares, so the common factor rstd is left
// out: the kernel writes gain * h as 16-bit terms and the quarter's sum of squares (Act::ss), and the GEMM that
// reads the row multiplies its outputs by rstd, which is the same product in another order.  PR as above.
template <int PR>
__global__ __launch_bounds__(256) void rmsnorm_part_kernel(NormArgs a) {
  __shared__ float sh[4];
  const int t = blockIdx.x, part = blockIdx.y;
  const int nv = a.d >> 2;
  const int nvp = (nv + NORM_PARTS - 1) / NORM_PARTS;        // float4 slices per part: at most 256 (host check)
  const int i = part * nvp + (int)threadIdx.x;
  const bool mine = (int)threadIdx.x < nvp && i < nv;
  const int ic = mine ? i : part * nvp < nv ? part * nvp : 0;   // clamped: loads are unconditional, stores masked
  float* hrow = a.h + (size_t)t * a.d;
  const int dt = a.x.dtype;
  f32x4 v = *reinterpret_cast<const f32x4*>(hrow + 4 * ic);
  const u32x2 gb = *reinterpret_cast<const u32x2*>(a.gain + 4 * ic);
  if (a.add) {
    for (int s0 = 0; s0 < a.n_planes; s0 += PR) {            // PR planes per round, added in plane order
      f32x4 p[PR];
#pragma unroll
      for (int q = 0; q < PR; ++q) {
        const int sc = s0 + q < a.n_planes ? s0 + q : a.n_planes - 1;
        p[q] = *reinterpret_cast<const f32x4*>(a.add + ((size_t)sc * a.T_total + t) * a.d + 4 * ic);
      }
#pragma unroll
      for (int q = 0; q < PR; ++q)
        if (s0 + q < a.n_planes) v += p[q];
    }
  }
  if (a.moe_y) {
    int pp[8];
    float pw[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const bool ok = k < a.top_k;
      pp[k] = ok ? a.pair_pos[t * a.top_k + k] : 0;
      pw[k] = ok ? a.topk_w[t * a.top_k + k] : 0.f;
    }
    f32x4 y[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) y[k] = *reinterpret_cast<const f32x4*>(a.moe_y + (size_t)pp[k] * a.d + 4 * ic);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < 8; ++k) acc += y[k] * pw[k];         // slot order k = 0..K-1; unused slots weigh 0
    v += acc;
  }
  float ss = 0.f;
  if (mine) {
    if (a.add || a.moe_y) *reinterpret_cast<f32x4*>(hrow + 4 * i) = v;
    ss = v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
  }
  const float tot = block_sum_256(ss, sh);
  if (threadIdx.x == 0) a.x.ss[(size_t)NORM_PARTS * t + part] = tot;
  if (!mine) return;
  f32x4 o;
  o[0] = v[0] * h16_to_f32((h16_t)(gb[0] & 0xFFFFu), dt);
  o[1] = v[1] * h16_to_f32((h16_t)(gb[0] >> 16), dt);
  o[2] = v[2] * h16_to_f32((h16_t)(gb[1] & 0xFFFFu), dt);
  o[3] = v[3] * h16_to_f32((h16_t)(gb[1] >> 16), dt);
  h16_t hi[4], lo[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) split_h16(o[e], hi[e], lo[e], dt);
  const int k = 4 * i;
  h16_t* xo = a.x.p + frag_act_offset(t, k & ~7, 0, a.x.mtiles(), a.x.planes) + (k & 7);
  u32x2 pk = {(uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16)};
  *reinterpret_cast<u32x2*>(xo) = pk;
  if (a.x.planes == 2) {
    u32x2 pk2 = {(uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16)};
    *reinterpret_cast<u32x2*>(xo + 512) = pk2;
  }
}

// grid (token, head group): each of the four waves owns one head; lane i < hd/2 owns the pair (i, i + hd/2).
// The form of short calls: decode steps and chunks of up to 1024 tokens, any number of split-K planes.
__global__ __launch_bounds__(256) void qk_rope_append_kernel(RopeArgs a) {
  const int t = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int hd = a.hd, half = hd >> 1, dt = a.q_out.dtype;
  const int n_heads = a.Hq + 2 * a.Hkv;
  const int h = blockIdx.y * 4 + wave;
  if (h >= n_heads) return;
  const int pos = a.tok_pos[t];
  const int seq = a.tok_seq[t];
  const bool live = a.tok_live[t] != 0;
  const size_t plane = (size_t)a.T * n_heads * hd;
  const float* src = a.qkv + ((size_t)t * n_heads + h) * hd;
  const bool act = lane < half;
  const int li = act ? lane : 0;

  float x0, x1;
  sum_head_planes(src, plane, a.n_planes, act, li, half, x0, x1);

  const bool is_q = h < a.Hq, is_k = !is_q && h < a.Hq + a.Hkv;
  int64_t blk = -1;
  if (live && !is_q) {
    int j = pos >> 4;
    if (j < a.max_blocks) blk = a.block_table[(size_t)seq * a.max_blocks + j];
    if (blk < 0 || blk >= a.n_blocks) blk = -1;   // bad table entry: drop the append instead of faulting
  }
  const int slot = pos & 15;

  if (is_q || is_k) {
    float c, s, y0, y1;
    const float2 cs = a.rope_cs[(size_t)t * half + li];
    c = cs.x; s = cs.y;
    head_norm_rope(x0, x1, is_q ? a.q_gain : a.k_gain, dt, hd, a.eps, act, lane, c, s, y0, y1);
    if (act) {
      if (is_q) {
        h16_t* dst = a.q_out.p + ((size_t)t * a.Hq + h) * hd;
        h16_t h0, l0, h1, l1;
        split_h16(y0, h0, l0, dt);
        split_h16(y1, h1, l1, dt);
        dst[lane] = h0;
        dst[lane + half] = h1;
        if (a.q_out.planes == 2) { dst[a.q_out.plane + lane] = l0; dst[a.q_out.plane + lane + half] = l1; }
      } else if (blk >= 0) {
        int kvh = h - a.Hq;
        h16_t* dst = a.pool_layer + (((size_t)blk * a.Hkv + kvh) * 2) * 16 * hd + (size_t)slot * hd;
        dst[lane] = f32_to_h16(y0, dt);
        dst[lane + half] = f32_to_h16(y1, dt);
      }
    }
  } else if (blk >= 0 && act) {   // value head: stored transposed, [hd][16]
    int kvh = h - a.Hq - a.Hkv;
    h16_t* dst = a.pool_layer + (((size_t)blk * a.Hkv + kvh) * 2 + 1) * 16 * hd;
    dst[(size_t)lane * 16 + slot] = f32_to_h16(x0, dt);
    dst[(size_t)(lane + half) * 16 + slot] = f32_to_h16(x1, dt);
  }
}

// Long calls (one plane): the kernel above spends its time issuing instructions for two elements per lane, so here
// 16 lanes share a head and a wave takes four heads of NT tokens.  Lane j of a head owns the pairs j + 16 k
// (k < HD / 32): summing its squares as (k = 0 with 2) + (1 with 3) and then across the 16 lanes is the butterfly
// of the 64-lane form with its first two levels done locally, and every other operation is per element, so both
// kernels give the same bits.  Neighbouring lanes exchange codes so that the 16-bit results leave as 32-bit stores.
template <int HD, int NT>
__global__ __launch_bounds__(256) void qk_rope_append_wide_kernel(RopeArgs a) {
  constexpr int half = HD / 2, PPL = HD / 32;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = lane & 15, odd = lane & 1;
  const int dt = a.q_out.dtype;
  const int n_heads = a.Hq + 2 * a.Hkv;
  const int h = (blockIdx.x * 4 + wave) * 4 + (lane >> 4);
  const bool head_ok = h < n_heads;
  const int hc = head_ok ? h : n_heads - 1;        // lanes past the last head repeat it and store nothing
  const bool is_q = hc < a.Hq, is_k = !is_q && hc < a.Hq + a.Hkv;
  const h16_t* gain = is_q ? a.q_gain : a.k_gain;  // both null or both set
  const bool normed = gain != nullptr && (is_q || is_k);

  float g0[PPL], g1[PPL];
#pragma unroll
  for (int k = 0; k < PPL; ++k) {
    g0[k] = normed ? h16_to_f32(gain[j + 16 * k], dt) : 1.f;
    g1[k] = normed ? h16_to_f32(gain[j + 16 * k + half], dt) : 1.f;
  }
  int tc[NT], pos[NT], seq[NT];
  bool live[NT];
  float x0[NT][PPL], x1[NT][PPL];
  float2 cs[NT][PPL];
#pragma unroll
  for (int i = 0; i < NT; ++i) {
    const int t = blockIdx.y * NT + i;
    tc[i] = t < a.T ? t : a.T - 1;                 // past the end: a repeated token, never stored
    pos[i] = a.tok_pos[tc[i]];
    seq[i] = a.tok_seq[tc[i]];
    live[i] = t < a.T && a.tok_live[tc[i]] != 0;
  }
#pragma unroll
  for (int i = 0; i < NT; ++i) {
    const float* src = a.qkv + ((size_t)tc[i] * n_heads + hc) * HD;
#pragma unroll
    for (int k = 0; k < PPL; ++k) {
      x0[i][k] = src[j + 16 * k];
      x1[i][k] = src[j + 16 * k + half];
      cs[i][k] = a.rope_cs[(size_t)tc[i] * half + j + 16 * k];
    }
  }
  int64_t blk[NT];
#pragma unroll
  for (int i = 0; i < NT; ++i) {
    blk[i] = -1;
    if (live[i] && !is_q && head_ok) {
      const int jb = pos[i] >> 4;
      if (jb < a.max_blocks) blk[i] = a.block_table[(size_t)seq[i] * a.max_blocks + jb];
      if (blk[i] < 0 || blk[i] >= a.n_blocks) blk[i] = -1;   // bad table entry: drop the append instead of faulting
    }
  }
#pragma unroll
  for (int i = 0; i < NT; ++i) {
    const int t = blockIdx.y * NT + i;
    if (t >= a.T) break;                           // uniform over the workgroup
    const int slot = pos[i] & 15;
    float u0[PPL], u1[PPL], p[PPL];
#pragma unroll
    for (int k = 0; k < PPL; ++k) {
      u0[k] = 0.f + x0[i][k];                      // the plane sum of the 64-lane form with one plane
      u1[k] = 0.f + x1[i][k];
      p[k] = __builtin_fmaf(u1[k], u1[k], u0[k] * u0[k]);
    }
    float ss = PPL == 4 ? (p[0] + p[2]) + (p[1] + p[3]) : p[0] + p[1];
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) ss += __shfl_xor(ss, o, WAVE);
    const float rstd = 1.0f / sqrtf(ss / (float)HD + a.eps);
    uint32_t mine[PPL], theirs[PPL];               // (large | small << 16) codes: mine to store, theirs to hand over
#pragma unroll
    for (int k = 0; k < PPL; ++k) {
      float v0 = u0[k], v1 = u1[k];
      if (normed) { v0 = v0 * rstd * g0[k]; v1 = v1 * rstd * g1[k]; }
      float y0 = v0, y1 = v1;
      if (is_q || is_k) {
        y0 = __builtin_fmaf(v0, cs[i][k].x, -(v1 * cs[i][k].y));
        y1 = __builtin_fmaf(v1, cs[i][k].x, v0 * cs[i][k].y);
      }
      h16_t h0, l0 = 0, h1, l1 = 0;
      if (is_q) { split_h16(y0, h0, l0, dt); split_h16(y1, h1, l1, dt); }
      else { h0 = f32_to_h16(y0, dt); h1 = f32_to_h16(y1, dt); }
      const uint32_t c0 = (uint32_t)h0 | ((uint32_t)l0 << 16), c1 = (uint32_t)h1 | ((uint32_t)l1 << 16);
      mine[k] = odd ? c1 : c0;                     // even lanes store the first half, odd lanes the second
      theirs[k] = __shfl_xor(odd ? c0 : c1, 1, WAVE);
    }
    if (!head_ok) continue;
    if (is_q || is_k) {
      h16_t* dst = nullptr;
      if (is_q) dst = a.q_out.p + ((size_t)t * a.Hq + hc) * HD;
      else if (blk[i] >= 0) dst = a.pool_layer + (((size_t)blk[i] * a.Hkv + (hc - a.Hq)) * 2) * 16 * HD + (size_t)slot * HD;
      if (dst) {
#pragma unroll
        for (int k = 0; k < PPL; ++k) {
          // even lane j: elements (j, j + 1) + 16 k of the first half; odd lane j: (j - 1, j) + 16 k of the second
          const uint32_t lo_lane = odd ? theirs[k] : mine[k], hi_lane = odd ? mine[k] : theirs[k];
          h16_t* d = dst + (odd ? half + j - 1 : j) + 16 * k;
          *reinterpret_cast<uint32_t*>(d) = (lo_lane & 0xFFFFu) | (hi_lane << 16);
          if (is_q && a.q_out.planes == 2)
            *reinterpret_cast<uint32_t*>(d + a.q_out.plane) = (lo_lane >> 16) | (hi_lane & 0xFFFF0000u);
        }
      }
    } else if (blk[i] >= 0) {                      // value head: stored transposed, [hd][16]
      h16_t* dst = a.pool_layer + (((size_t)blk[i] * a.Hkv + (hc - a.Hq - a.Hkv)) * 2 + 1) * 16 * HD;
#pragma unroll
      for (int k = 0; k < PPL; ++k) {
        dst[(size_t)(j + 16 * k) * 16 + slot] = f32_to_h16(u0[k], dt);
        dst[(size_t)(j + 16 * k + half) * 16 + slot] = f32_to_h16(u1[k], dt);
      }
    }
  }
}

__global__ void pack_weight_kernel(const h16_t* src, h16_t* dst, int N, int K) {
  // one thread per 8-element group of the packed layout
  const size_t g = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t total = packed_weight_elems(N, K) / 8;
  if (g >= total) return;
  const int lane = (int)(g & 63);
  const size_t frag = g >> 6;
  const int KS = K >> 4;
  const size_t in_group = frag % ((size_t)KS * W_GROUP);
  const int ks = (int)(in_group / W_GROUP);
  const int nt = (int)(frag / ((size_t)KS * W_GROUP)) * W_GROUP + (int)(in_group % W_GROUP);
  const int n = nt * 32 + (lane & 31), k = ks * 16 + 8 * (lane >> 5);
  u32x4 v = {0u, 0u, 0u, 0u};
  if (n < N) v = *reinterpret_cast<const u32x4*>(src + (size_t)n * K + k);
  *reinterpret_cast<u32x4*>(dst + g * 8) = v;
}

__global__ void pack_gate_up_kernel(const h16_t* gate, const h16_t* up, h16_t* dst, int F, int K) {
  const size_t g = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t total = packed_weight_elems(2 * F, K) / 8;
  if (g >= total) return;
  const int lane = (int)(g & 63);
  const size_t frag = g >> 6;
  const int KS = K >> 4;
  const size_t in_group = frag % ((size_t)KS * W_GROUP);
  const int ks = (int)(in_group / W_GROUP);
  const int nt = (int)(frag / ((size_t)KS * W_GROUP)) * W_GROUP + (int)(in_group % W_GROUP);
  const int r = lane & 31, k = ks * 16 + 8 * (lane >> 5);
  u32x4 v = {0u, 0u, 0u, 0u};
  if (nt * 16 < F) v = *reinterpret_cast<const u32x4*>((r < 16 ? gate : up) + (size_t)(nt * 16 + (r & 15)) * K + k);
  *reinterpret_cast<u32x4*>(dst + g * 8) = v;
}

__global__ void pack_activation_kernel(const h16_t* src, h16_t* dst, int T, int K) {
  const size_t g = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // (t, k/8) pairs
  const int kg = K >> 3;
  if (g >= (size_t)T * kg) return;
  const int t = (int)(g / kg), k = (int)(g % kg) * 8;
  u32x4 v = *reinterpret_cast<const u32x4*>(src + (size_t)t * K + k);
  *reinterpret_cast<u32x4*>(dst + frag_act_offset(t, k, 0, (T + 31) / 32, 1)) = v;
}

__global__ void sum_planes_kernel(const float* planes, int n_planes, size_t n, float* y) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float v = 0.f;
  for (int s = 0; s < n_planes; ++s) v += planes[(size_t)s * n + i];
  y[i] = v;
}

__global__ void kv_copy_kernel(h16_t* pool, int64_t n_blocks, size_t block_elems, const int32_t* src,
                               const int32_t* dst, int n) {
  // grid: (pairs, layers); 16-byte vector copy of one page
  int i = blockIdx.x, l = blockIdx.y;
  int64_t s = src[i], d = dst[i];
  if (s < 0 || s >= n_blocks || d < 0 || d >= n_blocks || s == d) return;
  const u32x4* sp = reinterpret_cast<const u32x4*>(pool + ((size_t)l * n_blocks + s) * block_elems);
  u32x4* dp = reinterpret_cast<u32x4*>(pool + ((size_t)l * n_blocks + d) * block_elems);
  size_t nv = block_elems / 8;
  for (size_t j = threadIdx.x; j < nv; j += blockDim.x) dp[j] = sp[j];
}

}  // namespace

hipError_t meta_decode(const TokenMeta& m, int n_seqs, const int32_t* ctx_lens, const uint8_t* finished,
                       const double* inv_freq, int head_dim, hipStream_t st) {
  hipLaunchKernelGGL(meta_decode_kernel, dim3(n_seqs), dim3(64), 0, st, m, n_seqs, ctx_lens, finished, inv_freq,
                     head_dim / 2);
  return hipGetLastError();
}

hipError_t meta_prefill(const TokenMeta& m, int n_seqs, int total_tokens, const int32_t* cu_seqlens,
                        const int32_t* ctx_lens, const uint8_t* sample_last, const double* inv_freq, int head_dim,
                        hipStream_t st) {
  hipLaunchKernelGGL(meta_prefill_kernel, dim3(1), dim3(1024), 0, st, m, n_seqs, total_tokens, cu_seqlens, ctx_lens,
                     sample_last);
  if (total_tokens > 0)
    hipLaunchKernelGGL(rope_table_kernel, dim3((total_tokens + 3) / 4), dim3(256), 0, st, m, total_tokens, inv_freq,
                       head_dim / 2);
  return hipGetLastError();
}

hipError_t embed_tokens(const h16_t* embed, int vocab, int d, const int32_t* tokens, const h16_t* input_embeds,
                        int T, float* h, int dtype, hipStream_t st) {
  hipLaunchKernelGGL(embed_kernel, dim3(T), dim3(256), 0, st, embed, vocab, d, tokens, input_embeds, h, dtype);
  return hipGetLastError();
}

template <int NV>
static void launch_rmsnorm(const NormArgs& a, hipStream_t st) {
  const int np = a.add ? a.n_planes : 0;
  if (np <= 4) hipLaunchKernelGGL((rmsnorm_kernel<NV, 4>), dim3(a.T), dim3(256), 0, st, a);
  else if (np <= 8 || NV == 4) hipLaunchKernelGGL((rmsnorm_kernel<NV, 8>), dim3(a.T), dim3(256), 0, st, a);
  else hipLaunchKernelGGL((rmsnorm_kernel<(NV < 4 ? NV : 1), 16>), dim3(a.T), dim3(256), 0, st, a);
}

// rows in quarters, the common factor left to the consumer: only where the output asks for it (Act::ss)
bool rmsnorm_in_parts(int d) { return (d >> 2) <= NORM_PARTS * 256; }

hipError_t rmsnorm(const NormArgs& a, hipStream_t st) {
  const int nv = a.d >> 2;                   // float4 slices of a row; 256 threads hold NV each
  if (a.x.ss) {
    if (a.rows || a.xf || !rmsnorm_in_parts(a.d)) return hipErrorInvalidValue;
    const int np = a.add ? a.n_planes : 0;
    const dim3 grid(a.T, NORM_PARTS);
    if (np <= 4) hipLaunchKernelGGL((rmsnorm_part_kernel<4>), grid, dim3(256), 0, st, a);
    else if (np <= 8) hipLaunchKernelGGL((rmsnorm_part_kernel<8>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((rmsnorm_part_kernel<16>), grid, dim3(256), 0, st, a);
    return hipGetLastError();
  }
  if (nv <= 256) launch_rmsnorm<1>(a, st);
  else if (nv <= 512) launch_rmsnorm<2>(a, st);
  else if (nv <= 768) launch_rmsnorm<3>(a, st);
  else launch_rmsnorm<4>(a, st);             // rows longer than 4096 elements loop
  return hipGetLastError();
}

hipError_t qk_rope_append(const RopeArgs& a, hipStream_t st) {
  const int n_heads = a.Hq + 2 * a.Hkv;
  if (a.T > 1024 && a.n_planes == 1 && (a.hd == 128 || a.hd == 64)) {
    const dim3 grid((n_heads + 15) / 16, (a.T + 3) / 4);
    if (a.hd == 128) hipLaunchKernelGGL((qk_rope_append_wide_kernel<128, 4>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((qk_rope_append_wide_kernel<64, 4>), grid, dim3(256), 0, st, a);
  } else {
    hipLaunchKernelGGL(qk_rope_append_kernel, dim3(a.T, (n_heads + 3) / 4), dim3(256), 0, st, a);
  }
  return hipGetLastError();
}

hipError_t pack_weight(const h16_t* src, h16_t* dst, int N, int K, hipStream_t st) {
  const size_t groups = packed_weight_elems(N, K) / 8;
  hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, st, src, dst, N, K);
  return hipGetLastError();
}

hipError_t pack_gate_up(const h16_t* gate, const h16_t* up, h16_t* dst, int F, int K, hipStream_t st) {
  const size_t groups = packed_weight_elems(2 * F, K) / 8;
  hipLaunchKernelGGL(pack_gate_up_kernel, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, st, gate, up, dst, F, K);
  return hipGetLastError();
}

hipError_t pack_activation(const h16_t* src, h16_t* dst, int T, int K, hipStream_t st) {
  const size_t groups = (size_t)T * (K / 8);
  hipLaunchKernelGGL(pack_activation_kernel, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, st, src, dst, T, K);
  return hipGetLastError();
}

hipError_t sum_planes(const float* planes, int n_planes, size_t n, float* y, hipStream_t st) {
  hipLaunchKernelGGL(sum_planes_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, planes, n_planes, n, y);
  return hipGetLastError();
}

hipError_t kv_copy_blocks(h16_t* pool, int64_t n_blocks, int n_layers, size_t block_elems, const int32_t* src,
                          const int32_t* dst, int n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(kv_copy_kernel, dim3(n, n_layers), dim3(256), 0, st, pool, n_blocks, block_elems, src, dst, n);
  return hipGetLastError();
}

}  // namespace rlx
