// Weight-streaming skinny GEMM for decode and chunked prefill (gfx950, MFMA bf16).
//
//   y[t, n] = sum_k x[t, k] * W[n, k]      x bf16 [T, K], W bf16 [N, K] row-major, fp32 accumulate
//
// Every weight byte is read exactly once per 32*MT tokens.  A workgroup owns a
// 32-row tile of W (two tiles, gate and up, in the SwiGLU form); its waves split
// the K range, each wave runs v_mfma_f32_32x32x16_bf16 with the weight rows as the
// A operand and 32 tokens as the B operand, and the partial tiles are summed
// through LDS in a fixed order (deterministic).  Optional split-K across
// workgroups writes partial planes that the consumer adds in plane order.
#include "kernels.h"

namespace rlx {

namespace {

constexpr int GEMM_WAVES = 4;
constexpr int GEMM_THREADS = GEMM_WAVES * WAVE;

struct GemmArgs {
  const bf16_t* x;        // [planes][T, ldx]: activations as a sum of `planes` bf16 terms
  size_t x_plane;         // elements between planes
  const int32_t* x_rows;  // optional gather: logical token t reads row x_rows[t]
  int ldx;
  const bf16_t* w[3];     // up to three stacked row segments
  int w_rows[3];          // rows per segment (multiples of 32 except the last)
  const bf16_t* w2;       // SwiGLU: the "up" matrix (same shape as w[0])
  int N, K, T;
  int ksteps_per_wave;    // k-steps (16 wide) per wave
  float* y;               // EPI_STORE: [splits][T][ldy]
  int ldy;
  bf16_t* act;            // EPI_SWIGLU: [planes][T][ldy]
  size_t act_plane;
  // LM-head epilogue
  float* logits;          // optional [T][N]
  float* part;            // [T][n_tiles][4] = max, sumexp, best score, best index (as float bits)
  const uint64_t* seeds;
  const float* temperature;
  const int32_t* sample_pos;  // absolute position of the token being drawn, per row
  // expert-grouped form: blockIdx.y is the expert, its rows are [group_off[e], group_off[e+1])
  const int32_t* group_off;
  size_t w_expert_stride;     // elements between consecutive experts' matrices
};

enum { EPI_STORE = 0, EPI_SWIGLU = 1, EPI_LMHEAD = 2 };

__device__ __forceinline__ const bf16_t* seg_row(const GemmArgs& a, int n) {
  // pointer to row n of the stacked weight, or nullptr past the end
  if (n >= a.N) return nullptr;
  int s = 0;
  while (n >= a.w_rows[s]) { n -= a.w_rows[s]; ++s; }
  return a.w[s] + (size_t)n * a.K;
}

// ---- Philox-4x32-10 (Salmon et al., SC'11), written from the published definition ----
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t (&out)[4]) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    uint32_t h0 = __umulhi(0xD2511F53u, c0), l0 = 0xD2511F53u * c0;
    uint32_t h1 = __umulhi(0xCD9E8D57u, c2), l1 = 0xCD9E8D57u * c2;
    uint32_t n0 = h1 ^ c1 ^ k0, n2 = h0 ^ c3 ^ k1;
    c0 = n0; c1 = l1; c2 = n2; c3 = l0;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Gumbel(0,1) from a 32-bit word: u = (R + 0.5) 2^-32, g = -log(-log u).  For the upper
// half of the range -log u is taken as -log1p(-(1 - u)) so that it stays accurate and positive.
__device__ __forceinline__ float gumbel_from_u32(uint32_t r) {
  float nl;
  if (r < 0x80000000u) {
    float u = ((float)r + 0.5f) * 2.3283064365386963e-10f;
    nl = -logf(u);
  } else {
    float w = ((float)(0xFFFFFFFFu - r) + 0.5f) * 2.3283064365386963e-10f;  // 1 - u
    nl = -log1pf(-w);
  }
  return -logf(nl);
}

template <int MT, int EPI, int PL>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_skinny_kernel(GemmArgs a) {
  constexpr int NW = (EPI == EPI_SWIGLU) ? 2 : 1;
  __shared__ float red[GEMM_WAVES][NW * MT][4][WAVE][4];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n0 = blockIdx.x * 32;
  const int t0 = blockIdx.z * (32 * MT);
  const int r32 = lane & 31, half = lane >> 5;
  int split = blockIdx.y;
  int row_base = 0;            // first logical row of this workgroup's row set
  if (a.group_off) {           // grouped: one expert per blockIdx.y, no split-K
    const int e = blockIdx.y;
    row_base = a.group_off[e];
    a.T = a.group_off[e + 1] - row_base;
    if (t0 >= a.T) return;     // uniform over the workgroup, before any barrier
    a.w[0] += (size_t)e * a.w_expert_stride;
    if (EPI == EPI_SWIGLU) a.w2 += (size_t)e * a.w_expert_stride;
    split = 0;
  }

  const bf16_t* wrow = seg_row(a, n0 + r32);
  const bf16_t* wrow2 = nullptr;
  if (EPI == EPI_SWIGLU) wrow2 = (n0 + r32 < a.N) ? a.w2 + (size_t)(n0 + r32) * a.K : nullptr;
  const bf16_t* xrow[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    int t = t0 + 32 * m + r32;
    if (t < a.T) {
      int row = a.x_rows ? a.x_rows[row_base + t] : row_base + t;
      xrow[m] = a.x + (size_t)row * a.ldx;
    } else {
      xrow[m] = nullptr;
    }
  }

  f32x16 acc[NW * MT];
#pragma unroll
  for (int i = 0; i < NW * MT; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;

  const int ks_begin = (split * GEMM_WAVES + wave) * a.ksteps_per_wave;
  const int ks_total = (a.K + 15) >> 4;
  int ks_end = ks_begin + a.ksteps_per_wave;
  if (ks_end > ks_total) ks_end = ks_total;

  constexpr int U = 4;
  for (int ks = ks_begin; ks < ks_end; ks += U) {
    bf16x8 wf[U], wf2[U], xf[U][MT][PL];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int k = (ks + u) * 16 + half * 8;
      bool ok = (ks + u < ks_end) && (k < a.K);
      wf[u] = (ok && wrow) ? load_bf16x8(wrow + k) : zero_bf16x8();
      if (EPI == EPI_SWIGLU) wf2[u] = (ok && wrow2) ? load_bf16x8(wrow2 + k) : zero_bf16x8();
#pragma unroll
      for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int p = 0; p < PL; ++p)
          xf[u][m][p] = (ok && xrow[m]) ? load_bf16x8(xrow[m] + p * a.x_plane + k) : zero_bf16x8();
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int p = PL - 1; p >= 0; --p) {   // small term first
          acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[u], xf[u][m][p], acc[m], 0, 0, 0);
          if (EPI == EPI_SWIGLU)
            acc[MT + m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf2[u], xf[u][m][p], acc[MT + m], 0, 0, 0);
        }
    }
  }

  // ---- sum the waves' partial tiles through LDS, fixed order 0..3 ----
#pragma unroll
  for (int i = 0; i < NW * MT; ++i)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      f32x4 v = {acc[i][4 * q], acc[i][4 * q + 1], acc[i][4 * q + 2], acc[i][4 * q + 3]};
      *reinterpret_cast<f32x4*>(&red[wave][i][q][lane][0]) = v;
    }
  __syncthreads();
  // wave w finishes register group q = w: weight rows n0 + 8w + 4*half + {0..3}, token r32 of each tile
  const int q = wave;
  const int nrow = n0 + 8 * q + 4 * half;
  f32x4 s[NW * MT];
#pragma unroll
  for (int i = 0; i < NW * MT; ++i) {
    s[i] = *reinterpret_cast<f32x4*>(&red[0][i][q][lane][0]);
#pragma unroll
    for (int w = 1; w < GEMM_WAVES; ++w) {
      f32x4 v = *reinterpret_cast<f32x4*>(&red[w][i][q][lane][0]);
      s[i] += v;
    }
  }

  if (EPI == EPI_STORE) {
#pragma unroll
    for (int m = 0; m < MT; ++m) {
      int t = t0 + 32 * m + r32;
      if (t < a.T) {
        float* dst = a.y + ((size_t)split * a.T + row_base + t) * a.ldy + nrow;
        if (nrow + 3 < a.N) {
          *reinterpret_cast<f32x4*>(dst) = s[m];
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (nrow + j < a.N) dst[j] = s[m][j];
        }
      }
    }
  } else if (EPI == EPI_SWIGLU) {
#pragma unroll
    for (int m = 0; m < MT; ++m) {
      int t = t0 + 32 * m + r32;
      if (t < a.T) {
        bf16_t* dst = a.act + (size_t)(row_base + t) * a.ldy + nrow;
        float o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float g = s[m][j], u = s[MT + m][j];
          o[j] = g / (1.f + __expf(-g)) * u;
        }
        bf16_t hi[4], lo[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) split_bf16(o[j], hi[j], lo[j]);
        if (nrow + 3 < a.N) {
          u32x2 p = {(uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16)};
          *reinterpret_cast<u32x2*>(dst) = p;
          if (PL == 2) {
            u32x2 q2 = {(uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16)};
            *reinterpret_cast<u32x2*>(dst + a.act_plane) = q2;
          }
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (nrow + j < a.N) {
              dst[j] = hi[j];
              if (PL == 2) dst[a.act_plane + j] = lo[j];
            }
        }
      }
    }
  } else {  // EPI_LMHEAD: per token, reduce this tile's 32 vocabulary rows to (max, sumexp, best, argbest)
    __shared__ float lm[GEMM_WAVES][MT][WAVE][4];
#pragma unroll
    for (int m = 0; m < MT; ++m) {
      int t = t0 + 32 * m + r32;
      float mx = -INFINITY, se = 0.f, best = -INFINITY;
      int besti = 0x7FFFFFFF;
      if (t < a.T) {
        float temp = a.temperature[t];
        float invt = temp > 0.f ? 1.f / temp : 1.f;
        uint64_t seed = a.seeds[t];
        uint32_t rnd[4];
        // nrow is a multiple of 4: one Philox block covers this lane's four vocabulary ids
        philox4x32_10((uint32_t)(nrow >> 2), (uint32_t)a.sample_pos[t], 0u, 0u, (uint32_t)seed,
                      (uint32_t)(seed >> 32), rnd);
        if (a.logits && nrow + 3 < a.N) {
          *reinterpret_cast<f32x4*>(a.logits + (size_t)t * a.N + nrow) = s[m];
        } else if (a.logits) {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (nrow + j < a.N) a.logits[(size_t)t * a.N + nrow + j] = s[m][j];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (nrow + j < a.N) {
            float z = s[m][j] * invt;
            float sc = temp > 0.f ? z + gumbel_from_u32(rnd[j]) : z;
            if (sc > best) { best = sc; besti = nrow + j; }   // ascending j: ties keep the smaller id
            float nm = fmaxf(mx, z);
            se = se * __expf(mx - nm) + __expf(z - nm);
            mx = nm;
          }
        }
      }
      lm[wave][m][lane][0] = mx; lm[wave][m][lane][1] = se;
      lm[wave][m][lane][2] = best; lm[wave][m][lane][3] = __int_as_float(besti);
    }
    __syncthreads();
    // threads 0..32*MT-1 merge the 8 row groups of their token in ascending row order
    if (threadIdx.x < 32 * MT) {
      int m = threadIdx.x >> 5, r = threadIdx.x & 31;
      int t = t0 + 32 * m + r;
      if (t < a.T) {
        float mx = -INFINITY, se = 0.f, best = -INFINITY;
        int besti = 0x7FFFFFFF;
#pragma unroll
        for (int g = 0; g < 8; ++g) {  // rows n0 + 4g .. : wave = g / 2, half = g & 1
          const float* p = lm[g >> 1][m][r + 32 * (g & 1)];
          float pm = p[0], ps = p[1], pb = p[2];
          int pi = __float_as_int(p[3]);
          if (pb > best) { best = pb; besti = pi; }
          if (pm > -INFINITY) {
            float nm = fmaxf(mx, pm);
            se = se * __expf(mx - nm) + ps * __expf(pm - nm);
            mx = nm;
          }
        }
        float* o = a.part + ((size_t)t * gridDim.x + blockIdx.x) * 4;
        o[0] = mx; o[1] = se; o[2] = best; o[3] = __int_as_float(besti);
      }
    }
  }
}

template <int EPI>
void launch_mt(const GemmArgs& a, dim3 grid_xy, int mt, int planes, hipStream_t st) {
  // tokens are covered by grid.z super-tiles of 32*MT
  if (mt == 1) {
    dim3 g(grid_xy.x, grid_xy.y, (a.T + 31) / 32);
    if (planes == 2) hipLaunchKernelGGL((gemm_skinny_kernel<1, EPI, 2>), g, dim3(GEMM_THREADS), 0, st, a);
    else hipLaunchKernelGGL((gemm_skinny_kernel<1, EPI, 1>), g, dim3(GEMM_THREADS), 0, st, a);
  } else {
    dim3 g(grid_xy.x, grid_xy.y, (a.T + 63) / 64);
    if (planes == 2) hipLaunchKernelGGL((gemm_skinny_kernel<2, EPI, 2>), g, dim3(GEMM_THREADS), 0, st, a);
    else hipLaunchKernelGGL((gemm_skinny_kernel<2, EPI, 1>), g, dim3(GEMM_THREADS), 0, st, a);
  }
}

int pick_splits(int n_tiles, int ksteps, int max_splits) {
  // enough workgroups to cover 256 CUs a few times over, at least 4 k-steps per wave
  int s = 1;
  while (s < max_splits && n_tiles * s < 1024 && ksteps / (GEMM_WAVES * (s * 2)) >= 4) s *= 2;
  return s;
}

}  // namespace

int gemm_max_splits() { return 8; }

int gemm_plan_splits(int N, int K, int max_splits) {
  return pick_splits((N + 31) / 32, (K + 15) / 16, max_splits);
}

hipError_t gemm_store(const LinearW& w, const Act& x, const int32_t* x_rows, int T, float* y, int ldy,
                      int splits, hipStream_t st) {
  GemmArgs a = {};
  a.x = x.p; a.x_plane = x.plane; a.x_rows = x_rows; a.ldx = x.ld;
  for (int i = 0; i < 3; ++i) { a.w[i] = w.seg[i]; a.w_rows[i] = w.rows[i]; }
  a.N = w.N; a.K = w.K; a.T = T;
  int ksteps = (w.K + 15) / 16;
  a.ksteps_per_wave = (ksteps + splits * GEMM_WAVES - 1) / (splits * GEMM_WAVES);
  a.y = y; a.ldy = ldy;
  launch_mt<EPI_STORE>(a, dim3((w.N + 31) / 32, splits), T > 32 ? 2 : 1, x.planes, st);
  return hipGetLastError();
}

hipError_t gemm_swiglu(const bf16_t* w_gate, const bf16_t* w_up, int F, int K, const Act& x, int T,
                       const Act& act, hipStream_t st) {
  GemmArgs a = {};
  a.x = x.p; a.x_plane = x.plane; a.ldx = x.ld;
  a.w[0] = w_gate; a.w_rows[0] = F; a.w2 = w_up;
  a.N = F; a.K = K; a.T = T;
  int ksteps = (K + 15) / 16;
  a.ksteps_per_wave = (ksteps + GEMM_WAVES - 1) / GEMM_WAVES;
  a.act = const_cast<bf16_t*>(act.p); a.act_plane = act.plane; a.ldy = act.ld;
  launch_mt<EPI_SWIGLU>(a, dim3((F + 31) / 32, 1), T > 32 ? 2 : 1, x.planes, st);
  return hipGetLastError();
}

hipError_t gemm_grouped_swiglu(const bf16_t* w_gate, const bf16_t* w_up, int E, int F, int K, const Act& x,
                               const int32_t* x_rows, const int32_t* group_off, int max_rows, const Act& act,
                               hipStream_t st) {
  GemmArgs a = {};
  a.x = x.p; a.x_plane = x.plane; a.x_rows = x_rows; a.ldx = x.ld;
  a.w[0] = w_gate; a.w_rows[0] = F; a.w2 = w_up;
  a.N = F; a.K = K; a.T = max_rows;
  a.ksteps_per_wave = ((K + 15) / 16 + GEMM_WAVES - 1) / GEMM_WAVES;
  a.act = const_cast<bf16_t*>(act.p); a.act_plane = act.plane; a.ldy = act.ld;
  a.group_off = group_off; a.w_expert_stride = (size_t)F * K;
  launch_mt<EPI_SWIGLU>(a, dim3((F + 31) / 32, E), max_rows > 32 ? 2 : 1, x.planes, st);
  return hipGetLastError();
}

hipError_t gemm_grouped_store(const bf16_t* w, int E, int N, int K, const Act& x,
                              const int32_t* group_off, int max_rows, float* y, hipStream_t st) {
  GemmArgs a = {};
  a.x = x.p; a.x_plane = x.plane; a.ldx = x.ld;
  a.w[0] = w; a.w_rows[0] = N;
  a.N = N; a.K = K; a.T = max_rows;
  a.ksteps_per_wave = ((K + 15) / 16 + GEMM_WAVES - 1) / GEMM_WAVES;
  a.y = y; a.ldy = N;
  a.group_off = group_off; a.w_expert_stride = (size_t)N * K;
  launch_mt<EPI_STORE>(a, dim3((N + 31) / 32, E), max_rows > 32 ? 2 : 1, x.planes, st);
  return hipGetLastError();
}

int lmhead_tiles(int vocab) { return (vocab + 31) / 32; }

hipError_t gemm_lmhead(const bf16_t* w_lm, int V, int K, const Act& x, int T, float* logits, float* part,
                       const uint64_t* seeds, const float* temperature, const int32_t* sample_pos,
                       hipStream_t st) {
  GemmArgs a = {};
  a.x = x.p; a.x_plane = x.plane; a.ldx = x.ld;
  a.w[0] = w_lm; a.w_rows[0] = V;
  a.N = V; a.K = K; a.T = T;
  int ksteps = (K + 15) / 16;
  a.ksteps_per_wave = (ksteps + GEMM_WAVES - 1) / GEMM_WAVES;
  a.logits = logits; a.part = part; a.seeds = seeds; a.temperature = temperature; a.sample_pos = sample_pos;
  launch_mt<EPI_LMHEAD>(a, dim3((V + 31) / 32, 1), T > 32 ? 2 : 1, x.planes, st);
  return hipGetLastError();
}

}  // namespace rlx
