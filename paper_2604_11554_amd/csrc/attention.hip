// Prefill attention over the paged 16-bit KV pool.  A workgroup takes ATTN_QTILE = 64 consecutive query positions
// of one sequence for NCT * NHG heads of one KV group: wave w owns the 16 positions q0 + 16 (w & 3) of the heads
// NCT (w >> 2) + {0 .. NCT-1} (a column tile per head, causal mask per column) and walks all keys itself, so there
// is no merge; the pages (32 keys per step) pass through LDS once for all waves, double buffered, one barrier per
// step.  Two waves share a SIMD, so one wave's softmax arithmetic runs under the other's matrix products.  K rows are padded by 16 bytes in
// LDS so that the 16 rows of a fragment read fall into different banks.  With two-term queries the small terms
// of a wave's query fragments live in LDS too (each lane re-reads what it wrote), the large ones in registers.
#include "attn_core.h"

namespace rlx {
namespace {

template <int HD, int NCT, int NHG, int PL, int FMT>
__global__ __launch_bounds__(256 * NHG) void attn_prefill_kernel(AttnArgs a) {
  constexpr int THREADS = 256 * NHG;
  constexpr int DT = HD / 16, KS = HD / 32;
  constexpr int KROW = HD + 8;                         // elements per K row in LDS
  constexpr int KPAGE = 16 * KROW, VPAGE = 16 * HD;    // elements of a page's K rows (padded) and of its V^T
  constexpr int PAGE_LDS = KPAGE + VPAGE, STAGE = 2 * PAGE_LDS;
  constexpr int PAGE_CHUNKS = 2 * 16 * HD / 8;         // 16-byte chunks of a page in the pool (K, then V^T)
  constexpr int NLOAD = (2 * PAGE_CHUNKS + THREADS - 1) / THREADS;   // chunks per thread and step
  extern __shared__ __align__(16) unsigned char lds_raw[];
  h16_t* lds_kv = reinterpret_cast<h16_t*>(lds_raw);                                   // [2][STAGE]
  u32x4* lds_q = reinterpret_cast<u32x4*>(lds_raw + (size_t)2 * STAGE * sizeof(h16_t)); // [waves][NCT * KS][64]

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c16 = lane & 15, g = lane >> 4;
  const int group = a.Hq / a.Hkv;

  if ((int)blockIdx.x >= a.n_qtiles[0]) return;      // uniform over the workgroup
  const int seq = a.qtile_seq[blockIdx.x];
  const int q0 = a.qtile_q0[blockIdx.x] + 16 * (wave & 3);  // this wave's first query position
  const int passes = (group + NCT * NHG - 1) / (NCT * NHG);
  const int kvh = blockIdx.y / passes;
  const int hbase = ((blockIdx.y % passes) * NHG + (wave >> 2)) * NCT;
  const int ctx = a.ctx_lens[seq];
  const int nq = a.cu_seqlens[seq + 1] - a.cu_seqlens[seq];
  const bool tile_live = q0 < nq && hbase < group;
  const int key_end = ctx + min(q0 + 16, nq);                                  // keys this wave's columns can see
  const int key_end_wg = ctx + min(a.qtile_q0[blockIdx.x] + ATTN_QTILE, nq);   // ... and the workgroup's last wave

  // ---- query fragments and per-column limits ----
  h16x8 qf[NCT][KS];                                 // large terms (the only ones when PL == 1)
  u32x4* my_q = lds_q + (size_t)(threadIdx.x >> 6) * NCT * KS * WAVE + lane;
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
    for (int ks = 0; ks < KS; ++ks) {
      const h16_t* src = a.q.p + ((size_t)trow[c] * a.Hq + head[c]) * HD + 32 * ks + 8 * g;
      qf[c][ks] = col_ok[c] ? load_h16x8(src) : zero_h16x8();
      if (PL == 2) my_q[(c * KS + ks) * WAVE] = col_ok[c] ? load_h16x8(src + a.q.plane) : zero_h16x8();
    }
  }
  auto q_term = [&](int p, int c, int ks) -> h16x8 {
    return p == 0 ? qf[c][ks] : __builtin_bit_cast(h16x8, my_q[(c * KS + ks) * WAVE]);
  };

  WaveState<HD, NCT> st;
  st.reset();

  const float scale = rsqrtf((float)HD);
  const int32_t* table = a.block_table + (size_t)seq * a.max_blocks;
  const int blk_end = (key_end_wg + 15) >> 4;        // exclusive
  const int n_pairs = (blk_end + 1) >> 1;
  const size_t page = (size_t)2 * 16 * HD;           // elements of one (block, kv head)

  // staging: chunk c = thread + 256 i of a step's two pages; (page, chunk of the page) -> pool address, LDS slot
  struct Staged { u32x4 v[NLOAD]; bool ok0, ok1; };
  auto stage_load = [&](int pi, Staged& r) {
    const int j0 = 2 * pi, j1 = j0 + 1;
    int64_t b0 = (j0 < blk_end && j0 < a.max_blocks) ? table[j0] : -1;
    int64_t b1 = (j1 < blk_end && j1 < a.max_blocks) ? table[j1] : -1;
    r.ok0 = b0 >= 0 && b0 < a.n_blocks;
    r.ok1 = b1 >= 0 && b1 < a.n_blocks;
    if (!r.ok0) b0 = 0;                                // keep the loads in bounds; scores are masked
    if (!r.ok1) b1 = b0;
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
      int c = (int)threadIdx.x + THREADS * i;
      if (c >= 2 * PAGE_CHUNKS) c = 2 * PAGE_CHUNKS - 1;   // more threads than chunks: a repeated load, not stored
      const int64_t b = c < PAGE_CHUNKS ? b0 : b1;
      r.v[i] = *reinterpret_cast<const u32x4*>(a.pool_layer + ((size_t)b * a.Hkv + kvh) * page + (size_t)(c % PAGE_CHUNKS) * 8);
    }
  };
  auto stage_store = [&](int buf, const Staged& r) {
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
      const int c = (int)threadIdx.x + THREADS * i;
      if (c >= 2 * PAGE_CHUNKS) continue;
      const int pg = c / PAGE_CHUNKS, w = c % PAGE_CHUNKS;   // w < PAGE_CHUNKS / 2: a chunk of the K rows
      const int off = w < PAGE_CHUNKS / 2 ? (w / (HD / 8)) * KROW + (w % (HD / 8)) * 8 : KPAGE + (w - PAGE_CHUNKS / 2) * 8;
      *reinterpret_cast<u32x4*>(lds_kv + buf * STAGE + pg * PAGE_LDS + off) = r.v[i];
    }
  };

  Staged sg;
  stage_load(0, sg);
  stage_store(0, sg);
  bool ok0 = sg.ok0, ok1 = sg.ok1;
  __syncthreads();
  for (int pi = 0; pi < n_pairs; ++pi) {             // n_pairs is uniform over the workgroup
    stage_load(pi + 1 < n_pairs ? pi + 1 : pi, sg);  // in flight while this step is multiplied
    const h16_t* kv = lds_kv + (pi & 1) * STAGE;
    if (tile_live && 32 * pi < key_end) {            // uniform over the wave: steps past its last column are skipped
      h16x8 k0[KS], k1[KS], vf[DT];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        k0[ks] = load_h16x8(kv + c16 * KROW + 32 * ks + 8 * g);
        k1[ks] = load_h16x8(kv + PAGE_LDS + c16 * KROW + 32 * ks + 8 * g);
      }
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
        vf[dt] = load_2x4(kv + KPAGE + (16 * dt + c16) * 16 + 4 * g, kv + PAGE_LDS + KPAGE + (16 * dt + c16) * 16 + 4 * g);
      pair_step<HD, NCT, PL, FMT>(st, k0, k1, vf, q_term, 32 * pi, 32 * pi + 16, ok0, ok1, key_end, pos_col, scale, g);
    }
    stage_store((pi + 1) & 1, sg);                   // the other buffer: its readers passed the last barrier
    ok0 = sg.ok0; ok1 = sg.ok1;
    __syncthreads();
  }
  if (!tile_live) return;
  st.finish_denominators();
#pragma unroll
  for (int c = 0; c < NCT; ++c)
    if (col_ok[c]) store_column<HD, NCT, PL, FMT>(st, c, a.o, trow[c], head[c], g);
}

}  // namespace

template <int HD, int PL, int FMT>
static void launch_prefill(const AttnArgs& a, hipStream_t st) {
  constexpr int NCT = 2, NHG = 2;                    // four heads of a KV group per workgroup, two per wave
  constexpr size_t kv_bytes = (size_t)2 * 2 * (16 * (HD + 8) + 16 * HD) * sizeof(h16_t);   // two stages of two pages
  constexpr size_t q_bytes = PL == 2 ? (size_t)4 * NHG * NCT * (HD / 32) * WAVE * 16 : 0;
  constexpr size_t lds = kv_bytes + q_bytes;
  static bool raised = false;                        // above the default limit of 64 KB per workgroup
  if (!raised) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_prefill_kernel<HD, NCT, NHG, PL, FMT>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    raised = true;
  }
  const int group = a.Hq / a.Hkv;
  const int passes = (group + NCT * NHG - 1) / (NCT * NHG);
  hipLaunchKernelGGL((attn_prefill_kernel<HD, NCT, NHG, PL, FMT>), dim3(a.max_qtiles, a.Hkv * passes), dim3(256 * NHG),
                     lds, st, a);
}

hipError_t attention_prefill(const AttnArgs& a, hipStream_t st) {
  const bool two = a.q.planes == 2;
  // formats built: bf16 with one or two terms, fp16 with one term (checked when the model is created)
  if (a.o.dtype == DT_F16) {
    if (a.hd == 128) launch_prefill<128, 1, DT_F16>(a, st);
    else launch_prefill<64, 1, DT_F16>(a, st);
  } else if (a.hd == 128) {
    if (two) launch_prefill<128, 2, DT_BF16>(a, st);
    else launch_prefill<128, 1, DT_BF16>(a, st);
  } else {
    if (two) launch_prefill<64, 2, DT_BF16>(a, st);
    else launch_prefill<64, 1, DT_BF16>(a, st);
  }
  return hipGetLastError();
}

}  // namespace rlx
