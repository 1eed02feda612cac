// MoE routing: router logits in fp32, softmax top-k with renormalised weights,
// capture of the chosen expert ids (the record Rollout Routing Replay consumes,
// paper Sec. 5.5), and a stable, deterministic grouping of (token, slot) pairs by expert.
#include "kernels.h"

namespace rlx {
namespace {

constexpr int MAX_E = 256;

// one workgroup per token: 4 waves take experts round-robin, lanes stride over d
__global__ __launch_bounds__(256) void moe_router_kernel(RouterArgs a) {
  __shared__ float logit[MAX_E];
  const int t = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float* x = a.xf + (size_t)t * a.d;
  for (int e = wave; e < a.E; e += 4) {
    const bf16_t* w = a.w_router + (size_t)e * a.d;
    float acc = 0.f;
    for (int k = lane * 8; k < a.d; k += 64 * 8) {
      u32x4 wv = *reinterpret_cast<const u32x4*>(w + k);
      f32x4 x0 = *reinterpret_cast<const f32x4*>(x + k);
      f32x4 x1 = *reinterpret_cast<const f32x4*>(x + k + 4);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float wl = __uint_as_float(wv[j] << 16), wh = __uint_as_float(wv[j] & 0xFFFF0000u);
        float xa = (j < 2) ? x0[2 * j] : x1[2 * j - 4];
        float xb = (j < 2) ? x0[2 * j + 1] : x1[2 * j - 3];
        acc += xa * wl;
        acc += xb * wh;
      }
    }
    acc = wave_sum(acc);
    if (lane == 0) logit[e] = acc;
  }
  __syncthreads();
  if (wave != 0) return;

  // wave 0: top-k by (logit descending, id ascending); lane holds ids lane, lane+64, ...
  float v[MAX_E / 64];
#pragma unroll
  for (int j = 0; j < MAX_E / 64; ++j) v[j] = (lane + 64 * j < a.E) ? logit[lane + 64 * j] : -INFINITY;
  float mx = -INFINITY;
#pragma unroll
  for (int j = 0; j < MAX_E / 64; ++j) mx = fmaxf(mx, v[j]);
  mx = wave_max(mx);
  float sel_e[8];
  int sel_i[8];
  float denom = 0.f;
  for (int k = 0; k < a.top_k; ++k) {
    float bv = -INFINITY; int bi = 0x7FFFFFFF;
#pragma unroll
    for (int j = 0; j < MAX_E / 64; ++j)
      if (v[j] > bv) { bv = v[j]; bi = lane + 64 * j; }      // ascending id within the lane
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      float ov = __shfl_xor(bv, o, WAVE);
      int oi = __shfl_xor(bi, o, WAVE);
      if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    sel_i[k] = bi;
    sel_e[k] = __expf(bv - mx);
    denom += sel_e[k];
    if ((bi & 63) == lane) {
#pragma unroll
      for (int j = 0; j < MAX_E / 64; ++j)
        if (j == (bi >> 6)) v[j] = -INFINITY;
    }
  }
  if (lane < a.top_k) {
    // softmax over all experts then renormalised over the chosen ones == softmax over the chosen logits
    int idx = 0; float w = 0.f;
    for (int k = 0; k < a.top_k; ++k)
      if (k == lane) { idx = sel_i[k]; w = sel_e[k] / denom; }
    a.topk_idx[t * a.top_k + lane] = idx;
    a.topk_w[t * a.top_k + lane] = w;
    if (a.routing_out && (!a.tok_live || a.tok_live[t]))
      a.routing_out[((size_t)t * a.n_layers + a.layer) * a.top_k + lane] = idx;
  }
}

__global__ __launch_bounds__(256) void moe_count_kernel(const int32_t* idx, int n_pairs, int32_t* counts) {
  __shared__ int sh[4];
  const int e = blockIdx.x;
  int c = 0;
  for (int p = threadIdx.x; p < n_pairs; p += 256) c += (idx[p] == e);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o, WAVE);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = c;
  __syncthreads();
  if (threadIdx.x == 0) counts[e] = sh[0] + sh[1] + sh[2] + sh[3];
}

// workgroup e writes its pairs, in pair order, at [off_e, off_e + count_e)
__global__ __launch_bounds__(256) void moe_scatter_kernel(const int32_t* idx, int n_pairs, int top_k, int E,
                                                          const int32_t* counts, int32_t* group_off,
                                                          int32_t* sorted_token, int32_t* pair_pos) {
  __shared__ int sh[4];
  __shared__ int base_sh;
  const int e = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int c = 0;
  for (int i = threadIdx.x; i < e; i += 256) c += counts[i];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o, WAVE);
  if (lane == 0) sh[wave] = c;
  __syncthreads();
  if (threadIdx.x == 0) {
    int off = sh[0] + sh[1] + sh[2] + sh[3];
    base_sh = off;
    group_off[e] = off;
    if (e == E - 1) group_off[E] = off + counts[e];
  }
  __syncthreads();
  int base = base_sh;
  for (int p0 = 0; p0 < n_pairs; p0 += 256) {
    int p = p0 + threadIdx.x;
    bool hit = p < n_pairs && idx[p] == e;
    unsigned long long bal = __ballot(hit);
    int before = __popcll(bal & ((1ull << lane) - 1ull));
    int wcount = __popcll(bal);
    __syncthreads();                       // previous iteration's reads of sh are done
    if (lane == 0) sh[wave] = wcount;
    __syncthreads();
    int woff = 0;
    for (int w = 0; w < wave; ++w) woff += sh[w];
    if (hit) {
      int pos = base + woff + before;
      sorted_token[pos] = p / top_k;
      pair_pos[p] = pos;
    }
    base += sh[0] + sh[1] + sh[2] + sh[3];
  }
}

}  // namespace

hipError_t moe_router(const RouterArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(moe_router_kernel, dim3(a.T), dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t moe_group(const int32_t* topk_idx, int T, int top_k, int E, int32_t* counts, int32_t* group_off,
                     int32_t* sorted_token, int32_t* pair_pos, hipStream_t st) {
  hipLaunchKernelGGL(moe_count_kernel, dim3(E), dim3(256), 0, st, topk_idx, T * top_k, counts);
  hipLaunchKernelGGL(moe_scatter_kernel, dim3(E), dim3(256), 0, st, topk_idx, T * top_k, top_k, E, counts, group_off,
                     sorted_token, pair_pos);
  return hipGetLastError();
}

}  // namespace rlx
