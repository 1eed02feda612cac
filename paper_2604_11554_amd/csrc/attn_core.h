// Pieces shared by the prefill and decode attention kernels (gfx950, MFMA 16x16x32 on bf16 or fp16 operands;
// FMT names the format of the pool and of the query / probability terms).
//
// Pool page of one (layer, block, kv head):  K[16 tokens][hd]  then  V^T[hd][16 tokens].
// The transposed V page makes both contractions read 8 or 16 contiguous bytes per lane:
//   S^T[token, col]  = K[token, :] . Q[col, :]          A = K page rows,  B = Q columns
//   O^T[d, col]     += V^T[d, tokens] . P[tokens, col]  A = V^T rows,     B = P (registers of S^T)
// A "column" is one (query position, query head).  The softmax statistics of a column live in
// the lanes that hold that column, so rescaling is lane-local; the max over keys is reduced
// across the four 16-lane groups with two shuffles.
#pragma once
#include "kernels.h"

namespace rlx {

__device__ __forceinline__ h16x8 load_2x4(const h16_t* p0, const h16_t* p1) {
  u32x2 a = *reinterpret_cast<const u32x2*>(p0);
  u32x2 b = *reinterpret_cast<const u32x2*>(p1);
  u32x4 v = {a[0], a[1], b[0], b[1]};
  return __builtin_bit_cast(h16x8, v);
}
// the same from pages that the launch reads once (decode attention)
__device__ __forceinline__ h16x8 load_2x4_stream(const h16_t* p0, const h16_t* p1) {
  u32x2 a = load_stream_8(p0);
  u32x2 b = load_stream_8(p1);
  u32x4 v = {a[0], a[1], b[0], b[1]};
  return __builtin_bit_cast(h16x8, v);
}

// running softmax state of NCT column tiles: lane holds column (lane & 15), rows d = 16 dt + 4 (lane >> 4) + {0..3}
template <int HD, int NCT>
struct WaveState {
  float m[NCT], l[NCT];
  f32x4 o[NCT][HD / 16];
  __device__ __forceinline__ void reset() {
#pragma unroll
    for (int c = 0; c < NCT; ++c) {
      m[c] = -INFINITY; l[c] = 0.f;
#pragma unroll
      for (int dt = 0; dt < HD / 16; ++dt) o[c][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
  }
  // sum the four lane groups' partial denominators of each column (once, after the last key)
  __device__ __forceinline__ void finish_denominators() {
#pragma unroll
    for (int c = 0; c < NCT; ++c) {
      l[c] += __shfl_xor(l[c], 16, WAVE);
      l[c] += __shfl_xor(l[c], 32, WAVE);
    }
  }
};

// The K fragments of two pages (tokens j0*16.. and j1*16..), the V^T fragments of the same 32 tokens and
// the query fragments are in registers; one online-softmax step over these 32 keys.
//   k0/k1[ks]: page rows (lane & 15), features 32 ks + 8 (lane >> 4) .. +8
//   vf[dt]:    V^T rows 16 dt + (lane & 15), tokens 4 (lane >> 4) .. +4 of page 0 then of page 1
//   qf(p, c, ks): query fragment of term p, column tile c: column (lane & 15), features 32 ks + 8 (lane >> 4) .. +8
// A key is visible to column c when its page is valid, key < key_end and key <= pos_col[c].
template <int HD, int NCT, int PL, int FMT, typename QF>
__device__ __forceinline__ void pair_step(WaveState<HD, NCT>& st, const h16x8 (&k0)[HD / 32],
                                          const h16x8 (&k1)[HD / 32], const h16x8 (&vf)[HD / 16], QF qf,
                                          int key_base0, int key_base1, bool ok0, bool ok1, int key_end,
                                          const int (&pos_col)[NCT], float scale, int g) {
  constexpr int DT = HD / 16, KS = HD / 32;
  f32x4 s0[NCT], s1[NCT];
#pragma unroll
  for (int c = 0; c < NCT; ++c) { s0[c] = f32x4{0.f, 0.f, 0.f, 0.f}; s1[c] = f32x4{0.f, 0.f, 0.f, 0.f}; }
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
#pragma unroll
    for (int c = 0; c < NCT; ++c)
#pragma unroll
      for (int p = PL - 1; p >= 0; --p) {   // small term first
        const h16x8 q = qf(p, c, ks);
        s0[c] = mfma_16x16x32<FMT>(k0[ks], q, s0[c]);
        s1[c] = mfma_16x16x32<FMT>(k1[ks], q, s1[c]);
      }

  h16x8 pf[PL][NCT];
#pragma unroll
  for (int c = 0; c < NCT; ++c) {
    float mx = -INFINITY;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      int key0 = key_base0 + 4 * g + v, key1 = key_base1 + 4 * g + v;
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
    h16_t ph[8], pl[8];
#pragma unroll
    for (int v = 0; v < 4; ++v) { split_h16<FMT>(p0[v], ph[v], pl[v]); split_h16<FMT>(p1[v], ph[4 + v], pl[4 + v]); }
    u32x4 pk = {(uint32_t)ph[0] | ((uint32_t)ph[1] << 16), (uint32_t)ph[2] | ((uint32_t)ph[3] << 16),
                (uint32_t)ph[4] | ((uint32_t)ph[5] << 16), (uint32_t)ph[6] | ((uint32_t)ph[7] << 16)};
    pf[0][c] = __builtin_bit_cast(h16x8, pk);
    if (PL == 2) {
      u32x4 pk2 = {(uint32_t)pl[0] | ((uint32_t)pl[1] << 16), (uint32_t)pl[2] | ((uint32_t)pl[3] << 16),
                   (uint32_t)pl[4] | ((uint32_t)pl[5] << 16), (uint32_t)pl[6] | ((uint32_t)pl[7] << 16)};
      pf[PL - 1][c] = __builtin_bit_cast(h16x8, pk2);
    }
  }
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int c = 0; c < NCT; ++c)
#pragma unroll
      for (int p = PL - 1; p >= 0; --p)
        st.o[c][dt] = mfma_16x16x32<FMT>(vf[dt], pf[p][c], st.o[c][dt]);
}

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

// Fixed-order tree merge of a workgroup's four waves, (0<-2, 1<-3) then 0<-1; the result is valid in wave 0.
// lds_o: [2][NCT * HD/16 * 64] f32x4, lds_ml: [2][NCT * 2 * 64] floats.  Every wave must call this.
template <int HD, int NCT>
__device__ __forceinline__ void merge_waves(WaveState<HD, NCT>& st, f32x4* lds_o, float* lds_ml, int wave, int lane) {
  constexpr int NO = NCT * (HD / 16) * WAVE, NM = NCT * 2 * WAVE;
  if (wave >= 2) store_to_lds<HD, NCT>(st, lds_ml + (wave - 2) * NM, lds_o + (wave - 2) * NO, lane);
  __syncthreads();
  if (wave < 2) merge_from_lds<HD, NCT>(st, lds_ml + wave * NM, lds_o + wave * NO, lane);
  __syncthreads();
  if (wave == 1) store_to_lds<HD, NCT>(st, lds_ml, lds_o, lane);
  __syncthreads();
  if (wave == 0) merge_from_lds<HD, NCT>(st, lds_ml, lds_o, lane);
}

// normalised column c of `st` -> 16-bit (hi, lo) terms at row `trow`, features head*HD + ..., fragment order
template <int HD, int NCT, int PL, int FMT>
__device__ __forceinline__ void store_column(const WaveState<HD, NCT>& st, int c, const Act& o, int trow, int head,
                                             int g) {
  const float inv = st.l[c] > 0.f ? 1.f / st.l[c] : 0.f;
  const int mtiles = o.mtiles();
#pragma unroll
  for (int dt = 0; dt < HD / 16; ++dt) {
    f32x4 v = st.o[c][dt] * inv;
    h16_t hi[4], lo[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) split_h16<FMT>(v[j], hi[j], lo[j]);
    const int col = head * HD + 16 * dt + 4 * g;   // feature index of the output projection's K
    h16_t* dst = o.p + frag_act_offset(trow, col & ~7, 0, mtiles, PL) + (col & 7);
    u32x2 p = {(uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16)};
    *reinterpret_cast<u32x2*>(dst) = p;
    if (PL == 2) {
      u32x2 p2 = {(uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16)};
      *reinterpret_cast<u32x2*>(dst + 512) = p2;
    }
  }
}

}  // namespace rlx
