// Prefill attention over the paged 16-bit KV pool: a tile is 16 consecutive query positions of one
// head (NCT heads of one KV group per workgroup), causal mask per column; the four waves of a
// workgroup take page pairs round-robin and are merged through LDS in a fixed order.
#include "attn_core.h"

namespace rlx {
namespace {

template <int HD, int NCT, int PL, int FMT>
__global__ __launch_bounds__(256) void attn_prefill_kernel(AttnArgs a) {
  constexpr int DT = HD / 16, KS = HD / 32;
  __shared__ f32x4 lds_o[2 * NCT * DT * WAVE];
  __shared__ float lds_ml[2 * NCT * 2 * WAVE];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c16 = lane & 15, g = lane >> 4;
  const int group = a.Hq / a.Hkv;

  if ((int)blockIdx.x >= a.n_qtiles[0]) return;
  const int seq = a.qtile_seq[blockIdx.x];
  const int q0 = a.qtile_q0[blockIdx.x];
  const int passes = (group + NCT - 1) / NCT;
  const int kvh = blockIdx.y / passes;
  const int hbase = (blockIdx.y % passes) * NCT;
  const int ctx = a.ctx_lens[seq];
  const int nq = a.cu_seqlens[seq + 1] - a.cu_seqlens[seq];
  const int key_end = ctx + min(q0 + 16, nq);

  // ---- query fragments and per-column limits ----
  h16x8 qf[PL][NCT][KS];
  int pos_col[NCT];
  bool col_ok[NCT];
  int trow[NCT], head[NCT];
#pragma unroll
  for (int c = 0; c < NCT; ++c) {
    head[c] = kvh * group + hbase + c;
    col_ok[c] = (hbase + c < group) && (q0 + c16 < nq);
    trow[c] = a.cu_seqlens[seq] + q0 + c16;
    pos_col[c] = ctx + q0 + c16;
#pragma unroll
    for (int p = 0; p < PL; ++p)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        qf[p][c][ks] = col_ok[c] ? load_h16x8(a.q.p + p * a.q.plane + ((size_t)trow[c] * a.Hq + head[c]) * HD +
                                               32 * ks + 8 * g)
                                 : zero_h16x8();
  }

  WaveState<HD, NCT> st;
  st.reset();

  const float scale = rsqrtf((float)HD);
  const int32_t* table = a.block_table + (size_t)seq * a.max_blocks;
  const int blk_end = (key_end + 15) >> 4;           // exclusive
  const int n_pairs = (blk_end + 1) >> 1;
  const size_t page = (size_t)2 * 16 * HD;           // elements of one (block, kv head)

  for (int pi = wave; pi < n_pairs; pi += 4) {
    const int j0 = 2 * pi, j1 = j0 + 1;
    const bool has1 = j1 < blk_end;
    int64_t b0 = (j0 < a.max_blocks) ? table[j0] : -1;
    int64_t b1 = (has1 && j1 < a.max_blocks) ? table[j1] : -1;
    const bool ok0 = b0 >= 0 && b0 < a.n_blocks, ok1 = b1 >= 0 && b1 < a.n_blocks;
    if (!ok0) b0 = 0;                                  // keep the loads in bounds; scores are masked
    if (!ok1) b1 = b0;
    const h16_t* kp0 = a.pool_layer + ((size_t)b0 * a.Hkv + kvh) * page;
    const h16_t* kp1 = a.pool_layer + ((size_t)b1 * a.Hkv + kvh) * page;
    const h16_t* vp0 = kp0 + 16 * HD;
    const h16_t* vp1 = kp1 + 16 * HD;
    h16x8 k0[KS], k1[KS], vf[DT];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      k0[ks] = load_h16x8(kp0 + c16 * HD + 32 * ks + 8 * g);
      k1[ks] = load_h16x8(kp1 + c16 * HD + 32 * ks + 8 * g);
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
      vf[dt] = load_2x4(vp0 + (size_t)(16 * dt + c16) * 16 + 4 * g, vp1 + (size_t)(16 * dt + c16) * 16 + 4 * g);
    pair_step<HD, NCT, PL, FMT>(st, k0, k1, vf, [&](int p, int c, int ks) { return qf[p][c][ks]; }, j0 * 16, j1 * 16, ok0, ok1, key_end, pos_col, scale, g);
  }
  st.finish_denominators();
  merge_waves<HD, NCT>(st, lds_o, lds_ml, wave, lane);
  if (wave != 0) return;
#pragma unroll
  for (int c = 0; c < NCT; ++c)
    if (col_ok[c]) store_column<HD, NCT, PL, FMT>(st, c, a.o, trow[c], head[c], g);
}

}  // namespace

hipError_t attention_prefill(const AttnArgs& a, hipStream_t st) {
  constexpr int NCT = 4;
  const int group = a.Hq / a.Hkv;
  const int passes = (group + NCT - 1) / NCT;
  dim3 grid(a.max_qtiles, a.Hkv * passes);
  const bool two = a.q.planes == 2;
  // formats built: bf16 with one or two terms, fp16 with one term (checked when the model is created)
  if (a.o.dtype == DT_F16) {
    if (a.hd == 128) hipLaunchKernelGGL((attn_prefill_kernel<128, NCT, 1, DT_F16>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((attn_prefill_kernel<64, NCT, 1, DT_F16>), grid, dim3(256), 0, st, a);
  } else if (a.hd == 128) {
    if (two) hipLaunchKernelGGL((attn_prefill_kernel<128, NCT, 2, DT_BF16>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((attn_prefill_kernel<128, NCT, 1, DT_BF16>), grid, dim3(256), 0, st, a);
  } else {
    if (two) hipLaunchKernelGGL((attn_prefill_kernel<64, NCT, 2, DT_BF16>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((attn_prefill_kernel<64, NCT, 1, DT_BF16>), grid, dim3(256), 0, st, a);
  }
  return hipGetLastError();
}

}  // namespace rlx
