// Small memory-bound kernels: per-call token metadata, embedding gather, fused
// (residual add / split-K reduce / MoE combine) + RMSNorm, fused per-head q/k
// RMSNorm + rotary embedding + paged KV append, KV page copy.
#include "kernels.h"

namespace rlx {
namespace {

__global__ void meta_decode_kernel(TokenMeta m, int n, const int32_t* ctx, const uint8_t* fin) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  uint8_t live = fin[i] ? 0 : 1;
  m.tok_seq[i] = i;
  m.tok_pos[i] = ctx[i];
  m.tok_live[i] = live;
  m.sample_row[i] = i;
  m.sample_pos[i] = ctx[i] + 1;
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
  }
  for (int i = threadIdx.x; i < n_seqs; i += blockDim.x) {
    int len = cu[i + 1] - cu[i];
    m.sample_row[i] = len > 0 ? cu[i + 1] - 1 : 0;
    m.sample_pos[i] = ctx[i] + len;
    m.sample_on[i] = (sample_last[i] && len > 0) ? 1 : 0;
  }
  // query tiles of 16 positions, sequence by sequence (n_seqs <= 1024 per chunk of the scan)
  __syncthreads();
  int base = 0;
  for (int s0 = 0; s0 < n_seqs; s0 += 1024) {
    int cnt = min(1024, n_seqs - s0);
    if (threadIdx.x == 0) {
      int acc = base;
      for (int i = 0; i < cnt; ++i) {
        tile_base[i] = acc;
        acc += (cu[s0 + i + 1] - cu[s0 + i] + 15) >> 4;
      }
      tile_base[cnt] = acc;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < cnt; i += blockDim.x) {
      int nt = tile_base[i + 1] - tile_base[i];
      for (int j = 0; j < nt; ++j) {
        m.qtile_seq[tile_base[i] + j] = s0 + i;
        m.qtile_q0[tile_base[i] + j] = 16 * j;
      }
    }
    base = tile_base[cnt];
    __syncthreads();
  }
  if (threadIdx.x == 0) m.n_qtiles[0] = base;
}

__global__ void embed_kernel(const bf16_t* embed, int vocab, int d, const int32_t* tokens, const bf16_t* inj, float* h) {
  int t = blockIdx.x;
  int tok = tokens[t];
  const bf16_t* src;
  if (tok >= 0 && tok < vocab) src = embed + (size_t)tok * d;
  else if (tok < 0 && inj) src = inj + (size_t)t * d;
  else src = nullptr;   // out-of-range id: zero row rather than a stray read
  for (int i = threadIdx.x; i < d; i += blockDim.x) h[(size_t)t * d + i] = src ? bf16_to_f32(src[i]) : 0.f;
}

__device__ __forceinline__ float block_sum_256(float v, float* sh) {
  v = wave_sum(v);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = sh[0] + sh[1] + sh[2] + sh[3];
  __syncthreads();
  return r;
}

__global__ __launch_bounds__(256) void rmsnorm_kernel(NormArgs a) {
  __shared__ float sh[4];
  const int r = blockIdx.x;
  const int t = a.rows ? a.rows[r] : r;
  float* hrow = a.h + (size_t)t * a.d;
  const bool adding = (a.add != nullptr) || (a.moe_y != nullptr);
  float ss = 0.f;
  for (int i = threadIdx.x; i < a.d; i += 256) {
    float v = hrow[i];
    if (a.add) {
      for (int s = 0; s < a.n_planes; ++s) v += a.add[((size_t)s * a.T_total + t) * a.d + i];
    }
    if (a.moe_y) {
      float acc = 0.f;
      for (int k = 0; k < a.top_k; ++k) {
        int p = a.pair_pos[t * a.top_k + k];
        acc += a.topk_w[t * a.top_k + k] * a.moe_y[(size_t)p * a.d + i];
      }
      v += acc;
    }
    if (adding) hrow[i] = v;
    ss += v * v;
  }
  float tot = block_sum_256(ss, sh);
  float rstd = 1.0f / sqrtf(tot / (float)a.d + a.eps);
  const int mtiles = a.x.mtiles();
  for (int i = threadIdx.x; i < a.d; i += 256) {
    float v = hrow[i] * rstd * bf16_to_f32(a.gain[i]);   // own writes: visible to the same thread
    bf16_t hi, lo;
    split_bf16(v, hi, lo);
    bf16_t* xo = a.x.p + frag_act_offset(r, i & ~7, 0, mtiles, a.x.planes) + (i & 7);
    xo[0] = hi;
    if (a.x.planes == 2) xo[512] = lo;
    if (a.xf) a.xf[(size_t)r * a.d + i] = v;
  }
}

// one workgroup per token, waves take heads round-robin; lane i < hd/2 owns the pair (i, i + hd/2)
__global__ __launch_bounds__(256) void qk_rope_append_kernel(RopeArgs a) {
  const int t = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int hd = a.hd, half = hd >> 1;
  const int n_heads = a.Hq + 2 * a.Hkv;
  const int pos = a.tok_pos[t];
  const int seq = a.tok_seq[t];
  const bool live = a.tok_live[t] != 0;
  const float* row = a.qkv + (size_t)t * n_heads * hd;
  const size_t plane = (size_t)a.T * n_heads * hd;

  float c = 1.f, s = 0.f;
  if (lane < half) {
    double ang = (double)pos * a.inv_freq[lane];
    double sd, cd;
    sincos(ang, &sd, &cd);
    c = (float)cd; s = (float)sd;
  }
  int64_t blk = -1;
  if (live) {
    int j = pos >> 4;
    if (j < a.max_blocks) blk = a.block_table[(size_t)seq * a.max_blocks + j];
    if (blk < 0 || blk >= a.n_blocks) blk = -1;   // bad table entry: drop the append instead of faulting
  }
  const int slot = pos & 15;

  for (int h = wave; h < n_heads; h += 4) {
    const float* src = row + (size_t)h * hd;
    float x0 = 0.f, x1 = 0.f;
    if (lane < half) {
      for (int p = 0; p < a.n_planes; ++p) {
        x0 += src[p * plane + lane];
        x1 += src[p * plane + lane + half];
      }
    }
    const bool is_q = h < a.Hq, is_k = !is_q && h < a.Hq + a.Hkv;
    if (is_q || is_k) {
      const bf16_t* gain = is_q ? a.q_gain : a.k_gain;
      if (gain) {
        float ss = wave_sum(x0 * x0 + x1 * x1);
        float rstd = 1.0f / sqrtf(ss / (float)hd + a.eps);
        if (lane < half) {
          x0 = x0 * rstd * bf16_to_f32(gain[lane]);
          x1 = x1 * rstd * bf16_to_f32(gain[lane + half]);
        }
      }
      float y0 = x0 * c - x1 * s, y1 = x1 * c + x0 * s;
      if (lane < half) {
        if (is_q) {
          bf16_t* dst = a.q_out.p + ((size_t)t * a.Hq + h) * hd;
          bf16_t h0, l0, h1, l1;
          split_bf16(y0, h0, l0);
          split_bf16(y1, h1, l1);
          dst[lane] = h0;
          dst[lane + half] = h1;
          if (a.q_out.planes == 2) { dst[a.q_out.plane + lane] = l0; dst[a.q_out.plane + lane + half] = l1; }
        } else if (blk >= 0) {
          int kvh = h - a.Hq;
          bf16_t* dst = a.pool_layer + (((size_t)blk * a.Hkv + kvh) * 2) * 16 * hd + (size_t)slot * hd;
          dst[lane] = f32_to_bf16(y0);
          dst[lane + half] = f32_to_bf16(y1);
        }
      }
    } else if (blk >= 0 && lane < half) {   // value head: stored transposed, [hd][16]
      int kvh = h - a.Hq - a.Hkv;
      bf16_t* dst = a.pool_layer + (((size_t)blk * a.Hkv + kvh) * 2 + 1) * 16 * hd;
      dst[(size_t)lane * 16 + slot] = f32_to_bf16(x0);
      dst[(size_t)(lane + half) * 16 + slot] = f32_to_bf16(x1);
    }
  }
}

__global__ void pack_weight_kernel(const bf16_t* src, bf16_t* dst, int N, int K) {
  // one thread per 8-element group of the packed layout
  const size_t g = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t total = packed_weight_elems(N, K) / 8;
  if (g >= total) return;
  const int lane = (int)(g & 63);
  const size_t frag = g >> 6;
  const int KS = K >> 4;
  const int ks = (int)(frag % KS);
  const int nt = (int)(frag / KS);
  const int n = nt * 32 + (lane & 31), k = ks * 16 + 8 * (lane >> 5);
  u32x4 v = {0u, 0u, 0u, 0u};
  if (n < N) v = *reinterpret_cast<const u32x4*>(src + (size_t)n * K + k);
  *reinterpret_cast<u32x4*>(dst + g * 8) = v;
}

__global__ void pack_activation_kernel(const bf16_t* src, bf16_t* dst, int T, int K) {
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

__global__ void kv_copy_kernel(bf16_t* pool, int64_t n_blocks, size_t block_elems, const int32_t* src,
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
                       hipStream_t st) {
  hipLaunchKernelGGL(meta_decode_kernel, dim3((n_seqs + 255) / 256), dim3(256), 0, st, m, n_seqs, ctx_lens, finished);
  return hipGetLastError();
}

hipError_t meta_prefill(const TokenMeta& m, int n_seqs, int total_tokens, const int32_t* cu_seqlens,
                        const int32_t* ctx_lens, const uint8_t* sample_last, hipStream_t st) {
  hipLaunchKernelGGL(meta_prefill_kernel, dim3(1), dim3(1024), 0, st, m, n_seqs, total_tokens, cu_seqlens, ctx_lens,
                     sample_last);
  return hipGetLastError();
}

hipError_t embed_tokens(const bf16_t* embed, int vocab, int d, const int32_t* tokens, const bf16_t* input_embeds,
                        int T, float* h, hipStream_t st) {
  hipLaunchKernelGGL(embed_kernel, dim3(T), dim3(256), 0, st, embed, vocab, d, tokens, input_embeds, h);
  return hipGetLastError();
}

hipError_t rmsnorm(const NormArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(rmsnorm_kernel, dim3(a.T), dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t qk_rope_append(const RopeArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(qk_rope_append_kernel, dim3(a.T), dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t pack_weight(const bf16_t* src, bf16_t* dst, int N, int K, hipStream_t st) {
  const size_t groups = packed_weight_elems(N, K) / 8;
  hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, st, src, dst, N, K);
  return hipGetLastError();
}

hipError_t pack_activation(const bf16_t* src, bf16_t* dst, int T, int K, hipStream_t st) {
  const size_t groups = (size_t)T * (K / 8);
  hipLaunchKernelGGL(pack_activation_kernel, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, st, src, dst, T, K);
  return hipGetLastError();
}

hipError_t sum_planes(const float* planes, int n_planes, size_t n, float* y, hipStream_t st) {
  hipLaunchKernelGGL(sum_planes_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, planes, n_planes, n, y);
  return hipGetLastError();
}

hipError_t kv_copy_blocks(bf16_t* pool, int64_t n_blocks, int n_layers, size_t block_elems, const int32_t* src,
                          const int32_t* dst, int n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(kv_copy_kernel, dim3(n, n_layers), dim3(256), 0, st, pool, n_blocks, block_elems, src, dst, n);
  return hipGetLastError();
}

}  // namespace rlx
