// Last stage of a step: merge the LM-head tiles' (max, sumexp, best perturbed score,
// argbest) partials in tile order, apply teacher forcing and the length cap, score the
// emitted token (log-softmax of the temperature-scaled logits) and update the
// per-sequence state (token, cached length, finished flag).
#include "kernels.h"

namespace rlx {
namespace {

struct Part { float m, s, best; int besti; };

// Equal perturbed scores go to the smaller token id whatever the order of the merges.
__device__ __forceinline__ Part part_merge(Part a, Part b) {
  Part r;
  float mn = fmaxf(a.m, b.m);
  float ea = (a.m == -INFINITY) ? 0.f : __expf(a.m - mn);
  float eb = (b.m == -INFINITY) ? 0.f : __expf(b.m - mn);
  r.m = mn; r.s = a.s * ea + b.s * eb;
  const bool take_b = b.best > a.best || (b.best == a.best && b.besti < a.besti);
  r.best = take_b ? b.best : a.best;
  r.besti = take_b ? b.besti : a.besti;
  return r;
}

__global__ __launch_bounds__(256) void sample_finalize_kernel(FinalizeArgs a) {
  __shared__ Part sh[256];
  __shared__ float dsh[4];
  const int r = blockIdx.x;
  if (a.score && (a.forced[r] < 0 || a.forced[r] >= a.vocab)) {   // nothing to score at this position
    if (threadIdx.x == 0) a.out_logprobs[r] = 0.f;
    return;
  }
  const bool on = a.score || a.sample_on[r] != 0;
  if (!on) {                                  // inert row
    if (threadIdx.x == 0) {
      a.out_tokens[r] = a.pad;
      a.out_logprobs[r] = 0.f;
      if (a.out_sampled) a.out_sampled[r] = -1;
      if (!a.is_decode) a.finished[r] = 0;
    }
    return;
  }
  // thread t takes tiles t, t + 256, ... (one 16-byte record each, eight loads in flight), merged in
  // ascending order; then a fixed binary tree over the threads
  Part p = {-INFINITY, 0.f, -INFINITY, 0x7FFFFFFF};
  const f32x4* base = reinterpret_cast<const f32x4*>(a.part + (size_t)r * a.n_tiles * 4);
  for (int t0 = 0; t0 < a.n_tiles; t0 += 8 * 256) {
    f32x4 q[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int tile = t0 + u * 256 + (int)threadIdx.x;
      q[u] = base[tile < a.n_tiles ? tile : a.n_tiles - 1];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (t0 + u * 256 + (int)threadIdx.x < a.n_tiles) {
        Part b = {q[u][0], q[u][1], q[u][2], __float_as_int(q[u][3])};
        p = part_merge(p, b);
      }
  }
  sh[threadIdx.x] = p;
  __syncthreads();
  for (int stride = 1; stride < 256; stride <<= 1) {
    if ((threadIdx.x % (2 * stride)) == 0) sh[threadIdx.x] = part_merge(sh[threadIdx.x], sh[threadIdx.x + stride]);
    __syncthreads();
  }
  p = sh[0];
  const float lse = p.m + logf(p.s);
  const int sampled = p.besti;
  int tok = sampled;
  if (a.forced && a.forced[r] >= 0 && a.forced[r] < a.vocab) tok = a.forced[r];
  if (!a.score) {
    const int pos = a.sample_pos[r];
    if (pos >= a.max_ctx_len[r] - 1) tok = a.eos;
  }
  if (tok < 0 || tok >= a.vocab) tok = a.eos;   // cannot happen with a non-empty vocabulary; keeps the read in bounds

  // logit of the emitted token: the same 16-bit operands as the LM-head tiles, fp32 accumulate
  // (eight consecutive k are one 16-byte group in both layouts; a thread's loads of a round go out together)
  const int mtiles = a.x.mtiles();
  const int dt = a.x.dtype;
  const int ng = a.d >> 3;
  float acc = 0.f;
  for (int g0 = 0; g0 < ng; g0 += 2 * 256) {
    h16x8 xh[2], xl[2], wv[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int gi = g0 + u * 256 + (int)threadIdx.x;
      const int k = 8 * (gi < ng ? gi : ng - 1);
      const h16_t* x = a.x.p + frag_act_offset(r, k, 0, mtiles, a.x.planes);
      xh[u] = load_h16x8(x);
      xl[u] = a.x.planes == 2 ? load_h16x8(x + 512) : zero_h16x8();
      wv[u] = load_h16x8(a.w_lm + packed_weight_offset(tok, k, a.d));
    }
#pragma unroll
    for (int u = 0; u < 2; ++u)
      if (g0 + u * 256 + (int)threadIdx.x < ng) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int sh = 16 * (e & 1);
          float xv = h16_to_f32((h16_t)((xh[u][e >> 1] >> sh) & 0xFFFFu), dt);
          if (a.x.planes == 2) xv += h16_to_f32((h16_t)((xl[u][e >> 1] >> sh) & 0xFFFFu), dt);
          acc += xv * h16_to_f32((h16_t)((wv[u][e >> 1] >> sh) & 0xFFFFu), dt);
        }
      }
  }
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) dsh[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    float z = dsh[0] + dsh[1] + dsh[2] + dsh[3];
    float temp = a.temperature[a.row_seq ? a.row_seq[r] : r];
    float invt = temp > 0.f ? 1.f / temp : 1.f;
    a.out_logprobs[r] = z * invt - lse;
    if (a.score) return;
    a.out_tokens[r] = tok;
    if (a.out_sampled) a.out_sampled[r] = sampled;
    uint8_t fin = (tok == a.eos) ? 1 : 0;
    if (a.is_decode) {
      a.finished[r] = fin;          // the row was live at entry
      a.ctx_lens[r] += 1;
    } else {
      a.finished[r] = fin;
    }
  }
}

}  // namespace

hipError_t sample_finalize(const FinalizeArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(sample_finalize_kernel, dim3(a.n_rows), dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace rlx
