// Weight-streaming skinny GEMM for decode and chunked prefill (gfx950, MFMA 32x32x16 on bf16 or fp16 operands).
//
//   y[t, n] = sum_k x[t, k] * W[n, k]        fp32 accumulate
//
// Both operands are stored in MFMA fragment order (see common.h): every weight load of a wave
// reads one 1 KB block, eight full cache lines, nothing wasted, and the texture-address path is
// left free for the activations; the blocks of the four tiles of a workgroup alternate along k,
// so the workgroup as a whole streams one contiguous run.
// Each of the four waves of a workgroup owns one 32-row tile of W over the
// workgroup's K range and keeps two batches of weight fragments in flight in registers
// (HBM latency under load is several microseconds, so the bytes in flight per CU decide
// the achieved bandwidth).  The activations of the current K chunk are shared by the four
// waves through LDS (double buffered); the next chunk is fetched while the current one is
// multiplied.  No reduction across waves is needed.  Optional split-K across workgroups
// writes partial planes that the consumer adds in plane order (deterministic).
//
// Epilogues: plain store (q|k|v, o and down projections, expert down projection),
// SwiGLU (gate/up), LM head with fused log-sum-exp and Gumbel-max partials per 32-row tile.
#include <atomic>
#include <mutex>

#include "kernels.h"

namespace rlx {

namespace {

constexpr int GEMM_WAVES = 4;
constexpr int GEMM_THREADS = GEMM_WAVES * WAVE;

struct GemmArgs {
  const h16_t* x;        // fragment-ordered activations [T_x, K], `PL` planes
  int x_mtiles;           // ceil(T_x / 32)
  const float* x_ss;      // optional: activation row t lacks the factor rstd(t) of its norm (Act::ss); outputs take it
  float x_eps;
  const int32_t* x_rows;  // grouped gate/up: logical row r of the group reads activation row x_rows[r]
  const h16_t* w[3];     // packed weights, up to three stacked row segments
  int w_tiles[3];         // 32-row tiles per segment
  int N, K, T;
  int ksteps_per_split;   // k-steps (16 wide) per blockIdx.y
  float* y;               // EPI_STORE: [splits][T][ldy]
  int ldy;
  h16_t* act;            // EPI_SWIGLU: fragment-ordered [act_rows, N], `PL` planes
  int act_mtiles;
  // LM-head epilogue
  float* logits;          // optional [T][N]
  float* part;            // [T][n_tiles][4] = max, sumexp, best score, best index (as float bits)
  const uint64_t* seeds;
  const float* temperature;
  const int32_t* sample_pos;
  const int32_t* row_seq;     // optional: row t takes its temperature from entry row_seq[t] (scoring: token -> sequence)
  int draw;                   // 0: no Gumbel-max draw (scoring): the random words are not generated
  // expert-grouped form: blockIdx.y is the expert, its rows are [group_off[e], group_off[e+1])
  const int32_t* group_off;
  size_t w_expert_stride;     // packed elements between consecutive experts' matrices
  // expert-grouped decode form without a grouping pass: the kernel finds its expert's rows in the routing table itself
  const int32_t* route_idx;   // [n_pairs] expert of pair p = token * top_k + slot, or null (rows come from group_off)
  int n_pairs, top_k;
  int32_t* pub_group_off;     // [E + 1] written by this launch: first row of every expert in expert order
  int32_t* pub_pair_pos;      // [n_pairs] written by this launch: row of every pair in expert order
  // large-batch grouped form over a list of (expert, row tile) items: blockIdx.y is the item
  const int32_t* item_expert; // [grid y] expert of the item, -1: none
  const int32_t* item_tile;   // [grid y] tile of 256 rows of the expert's rows
};

enum { EPI_STORE = 0, EPI_SWIGLU = 1, EPI_LMHEAD = 2 };

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

// Gumbel(0,1) from a 32-bit word: u = (R + 0.5) 2^-32, g = -log(-log u).  The largest values of g, the ones that
// win the draw, come from u next to 1, so for the upper half of the range -log u is taken from w = 1 - u (exact
// from the integer): the series w + w^2/2 + w^3/3 + w^4/4 below 2^-6 (relative error w^4/5 < 2e-8), the
// hardware logarithm of 1 - w above (absolute error ~1e-7 on a value of at least 0.0156).  The hardware
// logarithm's absolute error of ~1e-7 is also what the other two logarithms carry (their arguments are not near
// 1 where it would matter, or their result is near 0 where it does not): g is within ~1e-5 of the exact value,
// three orders below the tolerance on the scores it is added to.  Branch-free: lanes of a wave hold both halves.
__device__ __forceinline__ float gumbel_from_u32(uint32_t r) {
  const bool upper = r >= 0x80000000u;
  const float u = ((float)r + 0.5f) * 2.3283064365386963e-10f;
  const float w = ((float)(0xFFFFFFFFu - r) + 0.5f) * 2.3283064365386963e-10f;   // 1 - u, meaningful when upper
  const float series = w * (1.f + w * (0.5f + w * (0.33333334f + w * 0.25f)));
  const float nl_hi = w < 0.015625f ? series : -__logf(1.f - w);
  const float nl = upper ? nl_hi : -__logf(u);
  return -__logf(nl);
}

// Epilogue of one 32-row weight tile `nt` over token tiles mt0 .. mt0 + MT - 1: lane holds token r32 of each token
// tile, rows n0 + 8q + 4*half + {0..3}, q = 0..3, of the accumulators.
// factor that the norm left out of activation row `tok` (Act::ss): the same expression as in the norm kernel
__device__ __forceinline__ f32x4 row_ss(const GemmArgs& a, int tok) {
  return *reinterpret_cast<const f32x4*>(a.x_ss + (size_t)NORM_PARTS * tok);
}
__device__ __forceinline__ float row_rstd(const GemmArgs& a, const f32x4& p) {
  return 1.0f / sqrtf(((p[0] + p[1]) + (p[2] + p[3])) / (float)a.K + a.x_eps);
}

// rs[m]: factor of the lane's activation row in token tile m (row_rstd, or 1), fetched by the caller before its main
// loop so that the round trip is not spent at the end of the kernel
template <int MT, int EPI, int PL, int FMT>
__device__ __forceinline__ void tile_epilogue(const GemmArgs& a, const f32x16 (&acc)[MT], int nt, int n_tiles, int mt0,
                                              int split, int row_base, int lane, const float (&rs)[MT]) {
  const int r32 = lane & 31, half = lane >> 5;
  const int n0 = nt * 32;
  if (EPI == EPI_STORE) {
#pragma unroll
    for (int m = 0; m < MT; ++m) {
      const int t = (mt0 + m) * 32 + r32;
      if (t >= a.T) continue;
      float* dst = a.y + ((size_t)split * a.T + row_base + t) * a.ldy;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int nrow = n0 + 8 * q + 4 * half;
        f32x4 v = {acc[m][4 * q], acc[m][4 * q + 1], acc[m][4 * q + 2], acc[m][4 * q + 3]};
        if (a.x_ss) v *= rs[m];
        if (nrow + 3 < a.N) {
          *reinterpret_cast<f32x4*>(dst + nrow) = v;
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (nrow + j < a.N) dst[nrow + j] = v[j];
        }
      }
    }
  } else if (EPI == EPI_SWIGLU) {
    // The packed matrix interleaves gate and up: rows 0..15 of a tile are gate rows of features
    // 16 nt .. 16 nt + 15, rows 16..31 the matching up rows, so a lane holds both halves of a pair
    // (register groups q and q + 2).  The output feature is the K index of the down projection.
    const int n_feat = a.N >> 1;
#pragma unroll
    for (int m = 0; m < MT; ++m) {
      const int t = (mt0 + m) * 32 + r32;
      if (t >= a.T) continue;
      const int orow = row_base + t;
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int feat = nt * 16 + 8 * q + 4 * half;   // four consecutive features inside one 8-group
        if (feat >= n_feat) continue;
        h16_t hi[4], lo[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float g = acc[m][4 * q + j], u = acc[m][4 * (q + 2) + j];
          if (a.x_ss) { g *= rs[m]; u *= rs[m]; }
          split_h16<FMT>(g / (1.f + __expf(-g)) * u, hi[j], lo[j]);
        }
        h16_t* dst = a.act + frag_act_offset(orow, feat & ~7, 0, a.act_mtiles, PL) + (feat & 7);
        u32x2 pk = {(uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16)};
        *reinterpret_cast<u32x2*>(dst) = pk;
        if (PL == 2) {
          u32x2 pk2 = {(uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16)};
          *reinterpret_cast<u32x2*>(dst + 512) = pk2;
        }
      }
    }
  } else {  // EPI_LMHEAD: per token, reduce this tile's 32 vocabulary rows to (max, sumexp, best, argbest)
#pragma unroll
    for (int m = 0; m < MT; ++m) {
      const int t = (mt0 + m) * 32 + r32;
      const bool ok = t < a.T;
      float mx = -INFINITY, se = 0.f, best = -INFINITY;
      int besti = 0x7FFFFFFF;
      if (ok) {
        const float temp = a.temperature[a.row_seq ? a.row_seq[t] : t];
        const float invt = temp > 0.f ? 1.f / temp : 1.f;
        const bool draw = a.draw != 0 && temp > 0.f;          // uniform over the launch when draw == 0
        const uint64_t seed = a.draw ? a.seeds[t] : 0;
        const uint32_t pos = a.draw ? (uint32_t)a.sample_pos[t] : 0u;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int nrow = n0 + 8 * q + 4 * half;  // multiple of 4: one Philox block covers the four ids
          if (nrow >= a.N) continue;
          uint32_t rnd[4] = {0u, 0u, 0u, 0u};
          if (a.draw) philox4x32_10((uint32_t)(nrow >> 2), pos, 0u, 0u, (uint32_t)seed, (uint32_t)(seed >> 32), rnd);
          f32x4 v = {acc[m][4 * q], acc[m][4 * q + 1], acc[m][4 * q + 2], acc[m][4 * q + 3]};
          if (a.logits) {
            if (nrow + 3 < a.N) {
              *reinterpret_cast<f32x4*>(a.logits + (size_t)t * a.N + nrow) = v;
            } else {
#pragma unroll
              for (int j = 0; j < 4; ++j)
                if (nrow + j < a.N) a.logits[(size_t)t * a.N + nrow + j] = v[j];
            }
          }
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            if (nrow + j < a.N) {
              const float z = v[j] * invt;
              const float sc = draw ? z + gumbel_from_u32(rnd[j]) : z;
              if (sc > best) { best = sc; besti = nrow + j; }   // ascending ids: ties keep the smaller one
              const float nm = fmaxf(mx, z);
              se = se * __expf(mx - nm) + __expf(z - nm);
              mx = nm;
            }
          }
        }
      }
      // merge the two half-waves (rows 8q+0..3 and 8q+4..7) of the same token
      const float omx = __shfl_xor(mx, 32, WAVE), ose = __shfl_xor(se, 32, WAVE);
      const float obest = __shfl_xor(best, 32, WAVE);
      const int obesti = __shfl_xor(besti, 32, WAVE);
      if (obest > best || (obest == best && obesti < besti)) { best = obest; besti = obesti; }
      const float nm = fmaxf(mx, omx);
      if (nm > -INFINITY) {
        // fixed operand order (lower half first) so both half-waves compute the same bits
        const float lo_m = half ? omx : mx, lo_s = half ? ose : se, hi_m = half ? mx : omx, hi_s = half ? se : ose;
        se = lo_s * (lo_m == -INFINITY ? 0.f : __expf(lo_m - nm)) + hi_s * (hi_m == -INFINITY ? 0.f : __expf(hi_m - nm));
        mx = nm;
      }
      if (ok && half == 0) {
        float* o = a.part + ((size_t)t * n_tiles + nt) * 4;
        f32x4 pv = {mx, se, best, __int_as_float(besti)};
        *reinterpret_cast<f32x4*>(o) = pv;
      }
    }
  }
}

template <int MT, int PL>
struct Tiling {
  // k-steps per LDS chunk: 32 fragments (64 KB for both buffers) in general.  The 32-token two-term form, which
  // the expert-grouped decode GEMMs launch as thousands of workgroups, takes 24 (48 KB): with 64 KB only one
  // workgroup was resident per compute unit (in-kernel timestamps), with 48 KB two are (expert down GEMM -6 %).
  static constexpr int KC = (MT == 1 && PL == 2) ? 12 : ((32 / (MT * PL)) > 16 ? 16 : (32 / (MT * PL)));
  static constexpr int U = KC / 2;                                          // k-steps per weight batch (store form)
  static constexpr int FRAGS = KC * MT * PL;                                // 1 KB fragments per chunk
  static constexpr int PER_THREAD = FRAGS / GEMM_WAVES;                     // staged by each wave
  static constexpr int LDS_BYTES = 2 * FRAGS * 1024;
};

// ONCE: the launch reads every weight once (a single token tile per weight tile), so the weight loads are marked
// non-temporal; with several token tiles the later ones find the weights in the caches, and the mark would send
// them to memory again (decode steps of 129..256 tokens: down projection +10 % with the mark).
template <int MT, int EPI, int PL, int FMT, bool ONCE>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_skinny_kernel(GemmArgs a) {
  using TL = Tiling<MT, PL>;
  constexpr int KC = TL::KC, U = TL::U, FRAGS = TL::FRAGS, PT = TL::PER_THREAD;
  extern __shared__ __align__(16) unsigned char lds_raw[];
  u32x4* lds = reinterpret_cast<u32x4*>(lds_raw);   // [2][FRAGS][64 lanes]

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r32 = lane & 31, half = lane >> 5;
  const int mt0 = blockIdx.z * MT;                  // first 32-token tile of this workgroup
  int split = blockIdx.y;
  int row_base = 0;
  const bool grouped = a.group_off != nullptr;
  if (grouped) {
    const int e = blockIdx.y;
    row_base = a.group_off[e];
    a.T = a.group_off[e + 1] - row_base;
    if (mt0 * 32 >= a.T) return;                    // uniform over the workgroup, before any barrier
    a.w[0] += (size_t)e * a.w_expert_stride;
    split = 0;
  }

  // ---- this wave's weight tile ----
  // Every load below is unconditional (clamped address) and masked afterwards, so the main loop is
  // straight-line code and the hardware counters, not branches, order loads against their uses.
  const int KS = a.K >> 4;
  const int n_tiles = (a.N + 31) >> 5;
  const int nt = blockIdx.x * GEMM_WAVES + wave;
  const bool have_tile = nt < n_tiles;
  const h16_t* wp;
  {
    int lt = have_tile ? nt : 0;                    // a wave without a tile re-reads tile 0 and stores nothing
    const h16_t* base = a.w[0];                    // static member picks keep the pointers in the global space
    if (lt >= a.w_tiles[0]) {
      lt -= a.w_tiles[0];
      base = a.w[1];
      if (lt >= a.w_tiles[1]) { lt -= a.w_tiles[1]; base = a.w[2]; }
    }
    wp = base + packed_tile_offset(lt, KS) + lane * 8;
  }
  const int ks_b = split * a.ksteps_per_split;
  int ks_e = ks_b + a.ksteps_per_split;
  if (ks_e > KS) ks_e = KS;                          // the host never launches an empty split

  // ---- activation staging: each wave moves PT fragments of a chunk ----
  // fragment f of a chunk = (k-step f / (MT*PL), token tile (f / PL) % MT, plane f % PL)
  const h16_t* xsrc[MT];
  bool xok[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    if (grouped) {
      const int r = (mt0 + m) * 32 + r32;
      xok[m] = r < a.T;
      const int rr = xok[m] ? r : 0;
      const int row = a.x_rows ? a.x_rows[row_base + rr] : row_base + rr;
      xsrc[m] = a.x + frag_act_offset(row, 8 * half, 0, a.x_mtiles, PL);
    } else {
      xok[m] = mt0 + m < a.x_mtiles;
      const int mt = xok[m] ? mt0 + m : 0;
      xsrc[m] = a.x + (size_t)mt * PL * 512 + lane * 8;
    }
  }
  const size_t x_kstride = (size_t)a.x_mtiles * PL * 512;   // elements between consecutive k-steps
  // factor the norm left to this kernel's outputs (Act::ss), or 1: the sums are requested first of all, so that
  // no later wait has to sit through the weight batches for them, and turned into the factor after the first barrier
  f32x4 ssq[MT];
  float rs[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    const int t = (mt0 + m) * 32 + r32;
    ssq[m] = f32x4{1.f, 1.f, 1.f, 1.f};
    if (a.x_ss && !grouped) ssq[m] = row_ss(a, t < a.T ? t : 0);
  }
  __builtin_amdgcn_sched_barrier(0);
  // Fragment i of this wave belongs to the same token tile in every chunk.  With four token tiles the tile is picked
  // here, once, by comparing the wave number with constants, so that the arrays above are only ever indexed by
  // constants: the compiler turned the run-time choice among four into an indexed access, which put the arrays
  // into scratch memory with loads from it in the main loop (with two tiles it selects, in fewer registers).
  constexpr int NSEL = MT == 4 ? PT : 1;
  const h16_t* xsel[NSEL];
  bool oksel[NSEL];
  if (MT == 4) {
#pragma unroll
    for (int i = 0; i < NSEL; ++i) {
      xsel[i] = xsrc[0];
      oksel[i] = xok[0];
#pragma unroll
      for (int w = 0; w < GEMM_WAVES; ++w) {
        const int mw = ((w + GEMM_WAVES * i) / PL) % MT;      // a constant once both loops are unrolled
        if (wave == w) { xsel[i] = xsrc[mw]; oksel[i] = xok[mw]; }
      }
    }
  }
  auto tile_of = [&](int i, const h16_t*& src, bool& ok) {
    if (MT == 4) { src = xsel[i]; ok = oksel[i]; return; }
    const int m = ((wave + GEMM_WAVES * i) / PL) % MT;
    src = xsrc[0]; ok = xok[0];
#pragma unroll
    for (int mm = 1; mm < MT; ++mm)
      if (m == mm) { src = xsrc[mm]; ok = xok[mm]; }
  };
  auto stage_load = [&](int chunk, u32x4 (&r)[PT]) {
    const int ks0 = ks_b + chunk * KC;
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const int f = wave + GEMM_WAVES * i;
      const int ks = ks0 + f / (MT * PL), p = f % PL;
      const int ksc = ks < ks_e ? ks : ks_e - 1;
      const h16_t* src;
      bool ok;
      tile_of(i, src, ok);
      (void)ok;
      r[i] = *reinterpret_cast<const u32x4*>(src + (size_t)ksc * x_kstride + (size_t)p * 512);
    }
  };
  // the mask is applied when the fragments are written to LDS, long after the loads were issued
  auto stage_store = [&](int chunk, const u32x4 (&r)[PT]) {
    const int ks0 = ks_b + chunk * KC;
    const int buf = chunk & 1;
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const int f = wave + GEMM_WAVES * i;
      const int ks = ks0 + f / (MT * PL);
      const h16_t* src;
      bool ok;
      tile_of(i, src, ok);
      (void)src;
      const u32x4 z = {0u, 0u, 0u, 0u};
      lds[(buf * FRAGS + f) * 64 + lane] = (ok && ks < ks_e) ? r[i] : z;
    }
  };

  // ---- weight batches ----
  auto load_w = [&](int ks0, u32x4 (&wf)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int ks = ks0 + u;
      const int ksc = ks < ks_e ? ks : ks_e - 1;   // clamped: always a valid block; masked when used
      wf[u] = ONCE ? load_stream_16(wp + (size_t)ksc * W_KSTRIDE) : *reinterpret_cast<const u32x4*>(wp + (size_t)ksc * W_KSTRIDE);
    }
  };

  f32x16 acc[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;

  // One batch of U k-steps.  The activation fragments of k-step u + 1 are read from LDS while the matrix cores
  // work on k-step u (two register sets): with one wave per SIMD nothing else would hide the LDS latency.
  auto compute = [&](int buf, int kk0, int ks0, const u32x4 (&wf)[U]) {
    u32x4 xq[2][MT * PL];
    auto fetch = [&](int u, u32x4 (&dst)[MT * PL]) {
#pragma unroll
      for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int p = 0; p < PL; ++p) dst[m * PL + p] = lds[(buf * FRAGS + ((kk0 + u) * MT + m) * PL + p) * 64 + lane];
    };
    fetch(0, xq[0]);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (u + 1 < U) fetch(u + 1, xq[(u + 1) & 1]);
      __builtin_amdgcn_sched_barrier(0);          // the reads above are issued before the multiplies below
      const bool ok = ks0 + u < ks_e;             // uniform; past the end the weights count as zero
      const u32x4 z = {0u, 0u, 0u, 0u};
      const h16x8 w1 = ok ? wf[u] : z;
#pragma unroll
      for (int p = PL - 1; p >= 0; --p)           // small term first; the MT products of a term are independent
#pragma unroll
        for (int m = 0; m < MT; ++m) acc[m] = mfma_32x32x16<FMT>(w1, xq[u & 1][m * PL + p], acc[m]);
    }
  };

  // Ring of R weight batches in registers: while batch b is multiplied, batches b+1 .. b+R-1 are in
  // flight.  A group of R batches spans R/NBC activation chunks; k-steps past the end are masked to zero.
  constexpr int R = 4;
  constexpr int NBC = KC / U;                       // batches per activation chunk (divides R)
  const int n_groups = (ks_e - ks_b + R * U - 1) / (R * U);
  u32x4 wr[R][U];
  u32x4 xr[PT];
  stage_load(0, xr);
#pragma unroll
  for (int r = 0; r < R - 1; ++r) load_w(ks_b + r * U, wr[r]);
  __builtin_amdgcn_sched_barrier(0);
  stage_store(0, xr);
  __syncthreads();
  // the factors are complete here (their loads are as old as the first chunk's); the empty statement keeps the
  // compiler from moving the fetch down to the epilogue, where it would cost a round trip at the end of the kernel
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    rs[m] = (a.x_ss && !grouped) ? row_rstd(a, ssq[m]) : 1.f;
    asm volatile("" : "+v"(rs[m]));
  }
  for (int g = 0; g < n_groups; ++g) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int b = g * R + r;
      const int c = g * (R / NBC) + r / NBC;
      if (r % NBC == 0) stage_load(c + 1, xr);
      load_w(ks_b + (b + R - 1) * U, wr[(r + R - 1) % R]);
      // keep the issue order: the loads above go out before the multiply below starts waiting
      __builtin_amdgcn_sched_barrier(0);
      compute(c & 1, (r % NBC) * U, ks_b + b * U, wr[r]);
      __builtin_amdgcn_sched_barrier(0);
      if (r % NBC == NBC - 1) {
        stage_store(c + 1, xr);
        __syncthreads();
      }
    }
  }
  if (!have_tile) return;
  tile_epilogue<MT, EPI, PL, FMT>(a, acc, nt, n_tiles, mt0, split, row_base, lane, rs);
}

// ---- expert-grouped decode form: up to 32 rows per expert, J tile groups per workgroup ----
// At decode an expert receives a handful of rows, and the skinny form above then spends a tenth of its time on
// the activations: every workgroup stages all K of the expert's rows for the 128 weight rows it owns, so the rows
// are fetched as often as the expert has tile groups, with gather loads that touch sixteen cache lines for eight
// useful rows (measured at the 30B-A3B shape: gate/up 154 us with the activation loads, 144 us without, 135 us for a
// kernel that only streams the same weights).  Here a workgroup takes J consecutive tile groups of one expert: wave w
// owns tile w of each of them, the activation chunk in LDS serves all J, and a workgroup lives J times as long, so
// that the routing look-up, the first chunk and the epilogue are paid a J-th as often.  With the interleaved weight
// layout the J groups are J contiguous runs of 4 KB per k-step.  Per accumulator the products come in the order of
// the skinny form (k ascending, small term first): the results are the same bits.
//
// A chunk is KC k-steps of activations in LDS; its weight batches are taken in the order (first half of the chunk:
// tile group 0 .. J-1, second half: 0 .. J-1), U = KC / 2 k-steps each, through a ring of R batches in registers.
// (Four groups per workgroup leave registers for 4 KB batches only, which was measured slower than one group.)
template <int J>
struct ExpertTiling {
  static constexpr int KC = 16, U = 8, NBC = KC / U;
  static constexpr int BPC = J * NBC;                    // weight batches per chunk
  static constexpr int R = (BPC % 4 == 0) ? 4 : 3;       // ring depth: divides BPC, so ring slots are static
  static_assert(BPC % R == 0, "ring depth must divide the batches of a chunk");
};

template <int J, int EPI, int PL, int FMT>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_expert_kernel(GemmArgs a) {
  using TL = ExpertTiling<J>;
  constexpr int KC = TL::KC, U = TL::U, BPC = TL::BPC, R = TL::R;
  constexpr int FRAGS = KC * PL, PT = FRAGS / GEMM_WAVES;
  extern __shared__ __align__(16) unsigned char lds_raw[];
  u32x4* lds = reinterpret_cast<u32x4*>(lds_raw);   // [2][FRAGS][64 lanes]

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r32 = lane & 31, half = lane >> 5;
  const int mt0 = blockIdx.z;                       // 32-row tile of the expert's rows
  const int e = blockIdx.y;
  int row_base, my_pair = -1;
  if (a.route_idx) {
    // No grouping pass: the workgroup reads the routing table (a few KB, the same for every workgroup of the launch)
    // and finds what a counting sort by expert would have told it: how many pairs go to experts before this one
    // (row_base), how many to this one, and which, in pair order.  Thread i looks at the pairs i * PPT .. + PPT - 1,
    // so thread order is pair order.  One round trip, as the look-up of the sorted lists was.  The first workgroup
    // of each expert publishes the result (first row per expert, row of every pair) for the kernels that follow.
    __shared__ int32_t route_sum[GEMM_WAVES][2];
    __shared__ int32_t route_rows[32];              // pairs of this workgroup's tile of the expert's rows
    const int ppt = (a.n_pairs + GEMM_THREADS - 1) / GEMM_THREADS;
    const int p0 = (int)threadIdx.x * ppt;
    int less = 0, eq = 0;
    for (int i = 0; i < ppt; ++i) {
      const int p = p0 + i;
      const int idx = p < a.n_pairs ? a.route_idx[p] : 0x7FFFFFFF;
      less += idx < e ? 1 : 0;
      eq += idx == e ? 1 : 0;
    }
    int incl = eq;                                  // inclusive prefix of the matches over the wave's lanes
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int v = __shfl_up(incl, o, WAVE);
      if (lane >= o) incl += v;
    }
    less = (int)wave_sum((float)less);              // at most 4096 pairs: exact in fp32
    if (lane == 63) { route_sum[wave][0] = less; route_sum[wave][1] = incl; }
    if (threadIdx.x < 32) route_rows[threadIdx.x] = -1;
    __syncthreads();
    row_base = 0;
    int n_rows = 0, before = 0;
#pragma unroll
    for (int w = 0; w < GEMM_WAVES; ++w) {
      row_base += route_sum[w][0];
      if (w < wave) before += route_sum[w][1];
      n_rows += route_sum[w][1];
    }
    a.T = n_rows;
    if (blockIdx.x == 0 && mt0 == 0 && threadIdx.x == 0) {   // also for an expert without rows
      a.pub_group_off[e] = row_base;
      if (e == (int)gridDim.y - 1) a.pub_group_off[e + 1] = row_base + n_rows;
    }
    if (mt0 * 32 >= a.T) return;                    // uniform over the workgroup
    int pos = before + incl - eq - mt0 * 32;        // place, inside this tile, of the thread's first match
    for (int i = 0; i < ppt; ++i) {
      const int p = p0 + i;
      if (p < a.n_pairs && a.route_idx[p] == e) {   // second look at the same few entries: cache hits
        if (pos >= 0 && pos < 32) route_rows[pos] = p;
        ++pos;
      }
    }
    __syncthreads();
    my_pair = route_rows[r32];                      // -1 past the expert's last row
    if (blockIdx.x == 0) {
      if (threadIdx.x < 32 && my_pair >= 0) a.pub_pair_pos[my_pair] = row_base + mt0 * 32 + r32;
    }
  } else {
    row_base = a.group_off[e];
    a.T = a.group_off[e + 1] - row_base;
    if (mt0 * 32 >= a.T) return;                    // uniform over the workgroup, before any barrier
  }
  const h16_t* wbase = a.w[0] + (size_t)e * a.w_expert_stride;

  const int KS = a.K >> 4;
  const int n_tiles = (a.N + 31) >> 5;
  // tile of this wave in tile group j: (blockIdx.x * J + j) * 4 + wave; consecutive groups lie KS * W_KSTRIDE apart
  const int nt0 = blockIdx.x * J * W_GROUP + wave;
  static_assert(W_GROUP == GEMM_WAVES, "a wave owns one tile of every interleaved group");
  const h16_t* wp = wbase + packed_tile_offset(nt0, KS) + lane * 8;
  const size_t group_stride = (size_t)KS * W_KSTRIDE;
  // a tile group past the end of the matrix is read as the last one that exists (cache hits) and never stored
  int jmax = ((n_tiles + W_GROUP - 1) / W_GROUP) - 1 - blockIdx.x * J;
  if (jmax > J - 1) jmax = J - 1;

  // ---- activation staging: each wave moves PT fragments of a chunk; fragment f = (k-step f / PL, plane f % PL) ----
  const int r = mt0 * 32 + r32;
  const bool xok = r < a.T;
  const h16_t* xsrc;
  float rs[1];
  f32x4 ssq;
  {
    const int rr = xok ? r : 0;
    int row;
    if (a.route_idx) row = my_pair >= 0 ? my_pair / a.top_k : 0;       // the pair's token
    else row = a.x_rows ? a.x_rows[row_base + rr] : row_base + rr;
    xsrc = a.x + frag_act_offset(row, 8 * half, 0, a.x_mtiles, PL);
    ssq = f32x4{1.f, 1.f, 1.f, 1.f};
    if (a.x_ss && a.route_idx) ssq = row_ss(a, row);              // the pair's token is the activation row
    __builtin_amdgcn_sched_barrier(0);
  }
  const size_t x_kstride = (size_t)a.x_mtiles * PL * 512;
  auto stage_load = [&](int chunk, u32x4 (&rg)[PT]) {
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const int f = wave + GEMM_WAVES * i;
      const int ks = chunk * KC + f / PL, p = f % PL;
      const int ksc = ks < KS ? ks : KS - 1;         // clamped: always a valid fragment; masked when stored
      rg[i] = *reinterpret_cast<const u32x4*>(xsrc + (size_t)ksc * x_kstride + (size_t)p * 512);
    }
  };
  auto stage_store = [&](int chunk, const u32x4 (&rg)[PT]) {
    const int buf = chunk & 1;
    const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const int f = wave + GEMM_WAVES * i;
      const int ks = chunk * KC + f / PL;
      lds[(buf * FRAGS + f) * 64 + lane] = (xok && ks < KS) ? rg[i] : z;
    }
  };

  // ---- weight batches: batch s of chunk c = tile group s % J, k-steps c * KC + (s / J) * U .. + U ----
  auto load_w = [&](int c, int s, u32x4 (&wf)[U]) {
    const int j = s % J;
    const h16_t* base = wp + (size_t)(j < jmax ? j : jmax) * group_stride;
    const int ks0 = c * KC + (s / J) * U;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int ks = ks0 + u;
      const int ksc = ks < KS ? ks : KS - 1;         // clamped: always a valid block; masked when used
      wf[u] = load_stream_16(base + (size_t)ksc * W_KSTRIDE);
    }
  };

  f32x16 acc[J];
#pragma unroll
  for (int j = 0; j < J; ++j)
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[j][q] = 0.f;

  auto compute = [&](int buf, int kk0, int ks0, const u32x4 (&wf)[U], f32x16& ac) {
    u32x4 xq[2][PL];
    auto fetch = [&](int u, u32x4 (&dst)[PL]) {
#pragma unroll
      for (int p = 0; p < PL; ++p) dst[p] = lds[(buf * FRAGS + (kk0 + u) * PL + p) * 64 + lane];
    };
    fetch(0, xq[0]);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (u + 1 < U) fetch(u + 1, xq[(u + 1) & 1]);
      __builtin_amdgcn_sched_barrier(0);          // the reads above are issued before the multiplies below
      const bool ok = ks0 + u < KS;               // uniform; past the end the weights count as zero
      const u32x4 z = {0u, 0u, 0u, 0u};
      const h16x8 w1 = ok ? wf[u] : z;
#pragma unroll
      for (int p = PL - 1; p >= 0; --p) ac = mfma_32x32x16<FMT>(w1, xq[u & 1][p], ac);   // small term first
    }
  };

  const int n_chunks = (KS + KC - 1) / KC;
  u32x4 wr[R][U];
  u32x4 xr[PT];
  stage_load(0, xr);
  __builtin_amdgcn_sched_barrier(0);                // the activation loads are older than every weight load
#pragma unroll
  for (int s = 0; s < R - 1; ++s) load_w(0, s, wr[s]);
  __builtin_amdgcn_sched_barrier(0);
  stage_store(0, xr);
  __syncthreads();
  rs[0] = (a.x_ss && a.route_idx) ? row_rstd(a, ssq) : 1.f;   // as in the skinny form: fetched first, finished here
  asm volatile("" : "+v"(rs[0]));
  for (int c = 0; c < n_chunks; ++c) {
    stage_load(c + 1, xr);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int s = 0; s < BPC; ++s) {
      // batch s + R - 1 of this chunk, or the first batches of the next one, goes out before batch s is multiplied
      const int sn = s + R - 1;
      if (sn < BPC) load_w(c, sn, wr[sn % R]); else load_w(c + 1, sn - BPC, wr[sn % R]);
      __builtin_amdgcn_sched_barrier(0);
      compute(c & 1, (s / J) * U, c * KC + (s / J) * U, wr[s % R], acc[s % J]);
      __builtin_amdgcn_sched_barrier(0);
    }
    stage_store(c + 1, xr);
    __syncthreads();
  }
#pragma unroll
  for (int j = 0; j < J; ++j) {
    const int nt = nt0 + j * W_GROUP;
    if (nt < n_tiles) tile_epilogue<1, EPI, PL, FMT>(a, reinterpret_cast<const f32x16(&)[1]>(acc[j]), nt, n_tiles, mt0, 0, row_base, lane, rs);
  }
}

// ---- large-batch form (more than 128 tokens): 256 weight rows x 256 tokens per workgroup of eight waves ----
// With 128-token tiles and one weight tile per wave every compute unit takes in 12 KB per k-step for 32 multiplies;
// here both operands pass through LDS (each weight fragment feeds the two token halves, each activation fragment the
// four row groups), 24 KB per k-step feed 128 multiplies, and two waves per SIMD hide each other's LDS latency.
// Wave w = (row group w & 3: weight tiles 2 (w & 3) + {0, 1}; token half w >> 2: token tiles 4 (w >> 2) + {0..3}).
// Per accumulator the order is the same as in the skinny form (k ascending, small activation term first), so both
// forms give the same bits.
constexpr int LG_WAVES = 8, LG_THREADS = LG_WAVES * WAVE, LG_TILES = 8;

template <int PL>
struct LargeTiling {
  static constexpr int KC = 2;                          // k-steps per stage (three were measured slower)
  static constexpr int WFR = KC * LG_TILES;             // weight fragments per stage
  static constexpr int XFR = KC * LG_TILES * PL;        // activation fragments per stage
  static constexpr int STAGE = WFR + XFR;
  static constexpr int LDS_BYTES = 2 * STAGE * 1024;
};

template <int EPI, int PL, int FMT>
__global__ __launch_bounds__(LG_THREADS) void gemm_large_kernel(GemmArgs a) {
  using TL = LargeTiling<PL>;
  constexpr int KC = TL::KC, WFR = TL::WFR, STAGE = TL::STAGE;
  extern __shared__ __align__(16) unsigned char lds_raw[];
  u32x4* lds = reinterpret_cast<u32x4*>(lds_raw);   // [2][STAGE][64 lanes]

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r32 = lane & 31, half = lane >> 5;
  const int wr = wave & 3, wt = wave >> 2;
  int mt_base = blockIdx.z * LG_TILES;
  int split = blockIdx.y;
  int row_base = 0;
  const bool grouped = a.group_off != nullptr;
  if (grouped) {
    int e = blockIdx.y;
    if (a.item_expert) {                            // the grid runs over the list of (expert, row tile) items
      e = a.item_expert[blockIdx.y];
      if (e < 0) return;                            // uniform over the workgroup
      mt_base = a.item_tile[blockIdx.y] * LG_TILES;
    }
    row_base = a.group_off[e];
    a.T = a.group_off[e + 1] - row_base;
    if (mt_base * 32 >= a.T) return;                // uniform over the workgroup, before any barrier
    a.w[0] += (size_t)e * a.w_expert_stride;
    split = 0;
  }
  const int KS = a.K >> 4;
  const int n_tiles = (a.N + 31) >> 5;
  const int nt_base = blockIdx.x * LG_TILES;

  // ---- staging duties: wave w copies weight tile nt_base + w and token tile mt_base + w of every stage ----
  const h16_t* wp;
  int w_kstride = W_KSTRIDE;
  {
    int lt = nt_base + wave;
    if (lt >= n_tiles) { lt = 0; w_kstride = 0; }   // no such tile: one cached block, its products are never stored
    const h16_t* base = a.w[0];
    if (lt >= a.w_tiles[0]) {
      lt -= a.w_tiles[0];
      base = a.w[1];
      if (lt >= a.w_tiles[1]) { lt -= a.w_tiles[1]; base = a.w[2]; }
    }
    wp = base + packed_tile_offset(lt, KS) + lane * 8;
  }
  // a token row past the end reads row 0 / tile 0: a token's row only reaches its own outputs, which are not stored
  const h16_t* xsrc;
  if (grouped) {
    const int r = (mt_base + wave) * 32 + r32;
    const int rr = r < a.T ? r : 0;
    const int row = a.x_rows ? a.x_rows[row_base + rr] : row_base + rr;
    xsrc = a.x + frag_act_offset(row, 8 * half, 0, a.x_mtiles, PL);
  } else {
    const int mt = mt_base + wave < a.x_mtiles ? mt_base + wave : 0;
    xsrc = a.x + (size_t)mt * PL * 512 + lane * 8;
  }
  const size_t x_kstride = (size_t)a.x_mtiles * PL * 512;
  const int ks_b = split * a.ksteps_per_split;
  int ks_e = ks_b + a.ksteps_per_split;
  if (ks_e > KS) ks_e = KS;                          // the host never launches an empty split

  struct Staged { u32x4 w[KC]; u32x4 x[KC][PL]; };
  auto stage_load = [&](int s, Staged& r) {         // unconditional loads at clamped k-steps
#pragma unroll
    for (int kk = 0; kk < KC; ++kk) {
      const int ks = ks_b + s * KC + kk;
      const int ksc = ks < ks_e ? ks : ks_e - 1;
      r.w[kk] = *reinterpret_cast<const u32x4*>(wp + (size_t)ksc * w_kstride);
#pragma unroll
      for (int p = 0; p < PL; ++p) r.x[kk][p] = *reinterpret_cast<const u32x4*>(xsrc + (size_t)ksc * x_kstride + (size_t)p * 512);
    }
  };
  auto stage_store = [&](int s, const Staged& r) {  // a k-step past the end multiplies by zero weights
    const int buf = s & 1;
    const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int kk = 0; kk < KC; ++kk) {
      const bool ok = ks_b + s * KC + kk < ks_e;
      lds[(buf * STAGE + kk * LG_TILES + wave) * 64 + lane] = ok ? r.w[kk] : z;
#pragma unroll
      for (int p = 0; p < PL; ++p) lds[(buf * STAGE + WFR + (kk * LG_TILES + wave) * PL + p) * 64 + lane] = r.x[kk][p];
    }
  };

  f32x16 acc[2][4];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[j][m][q] = 0.f;

  // The products of a stage run in four phases of eight: (k-step 0, small term), (0, large), (1, small), (1, large).
  // Every phase first requests the fragments of the next one from LDS, so the matrix cores never wait for a read;
  // the stage's one barrier sits before its last phase, whose reads are the next stage's first fragments: the
  // next stage was written to the other buffer at the top of this iteration (from registers loaded one iteration
  // earlier), and the buffer written there was last read before the previous iteration's barrier.
  static_assert(KC == 2 && PL == 2, "the phase schedule below is written for two k-steps of two terms");
  auto read_w = [&](int buf, int kk, h16x8 (&wf)[2]) {
#pragma unroll
    for (int j = 0; j < 2; ++j) wf[j] = lds[(buf * STAGE + kk * LG_TILES + 2 * wr + j) * 64 + lane];
  };
  auto read_x = [&](int buf, int kk, int p, h16x8 (&xf)[4]) {
#pragma unroll
    for (int m = 0; m < 4; ++m) xf[m] = lds[(buf * STAGE + WFR + (kk * LG_TILES + 4 * wt + m) * PL + p) * 64 + lane];
  };
  auto products = [&](const h16x8 (&wf)[2], const h16x8 (&xf)[4]) {   // eight independent accumulators
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int m = 0; m < 4; ++m) acc[j][m] = mfma_32x32x16<FMT>(wf[j], xf[m], acc[j][m]);
  };
  // order of a phase's instructions: its LDS reads go out first, then its eight matrix-core instructions
#define reads_then_products(n_reads)                                   \
  __builtin_amdgcn_sched_group_barrier(0x100, (n_reads), 0);           \
  __builtin_amdgcn_sched_group_barrier(0x008, 8, 0)
  auto lds_barrier = [&]() {                          // LDS traffic only: global loads stay in flight across it
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  };

  const int n_stages = (ks_e - ks_b + KC - 1) / KC;
  Staged st;
  stage_load(0, st);
  stage_store(0, st);
  stage_load(1, st);
  __syncthreads();
  // A wave whose 128 tokens lie past the last row (the tail tile of an expert's rows, mostly) only stages: same
  // stores, loads and barriers, no fragments and no products, which leaves its SIMD to the wave it shares it with.
  if ((mt_base + 4 * wt) * 32 >= a.T) {             // uniform over the wave
    for (int s = 0; s < n_stages; ++s) {
      stage_store(s + 1, st);
      stage_load(s + 2, st);
      lds_barrier();
    }
    return;
  }
  h16x8 w0[2], w1[2], xa[4], xb[4];
  read_w(0, 0, w0);
  read_x(0, 0, 1, xa);
  for (int s = 0; s < n_stages; ++s) {
    const int buf = s & 1;
    stage_store(s + 1, st);                          // the other buffer: its readers passed the last barrier
    stage_load(s + 2, st);                           // in flight for one whole iteration
    __builtin_amdgcn_sched_barrier(0);
    read_x(buf, 0, 0, xb);
    products(w0, xa);                                // k-step 0, small term
    reads_then_products(4);
    __builtin_amdgcn_sched_barrier(0);
    read_w(buf, 1, w1);
    read_x(buf, 1, 1, xa);
    products(w0, xb);                                // k-step 0, large term
    reads_then_products(6);
    __builtin_amdgcn_sched_barrier(0);
    read_x(buf, 1, 0, xb);
    products(w1, xa);                                // k-step 1, small term
    reads_then_products(4);
    __builtin_amdgcn_sched_barrier(0);
    lds_barrier();                                   // stage s + 1 is complete; nobody reads stage s from here on
    __builtin_amdgcn_sched_barrier(0);
    read_w(buf ^ 1, 0, w0);
    read_x(buf ^ 1, 0, 1, xa);
    products(w1, xb);                                // k-step 1, large term
    reads_then_products(6);
    __builtin_amdgcn_sched_barrier(0);
  }
#undef reads_then_products
  // written out, not a loop: a loop that the compiler declines to unroll (it did with the LM-head epilogue inlined
  // twice) indexes the accumulators at run time, which moves all of them to scratch memory
  const int nt0 = nt_base + 2 * wr;
  float rs[4];                                       // rows of long calls come finished from the norm: no factor
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    const int t = (mt_base + 4 * wt + m) * 32 + r32;
    rs[m] = (a.x_ss && !grouped && t < a.T) ? row_rstd(a, row_ss(a, t)) : 1.f;
  }
  if (nt0 < n_tiles) tile_epilogue<4, EPI, PL, FMT>(a, acc[0], nt0, n_tiles, mt_base + 4 * wt, split, row_base, lane, rs);
  if (nt0 + 1 < n_tiles) tile_epilogue<4, EPI, PL, FMT>(a, acc[1], nt0 + 1, n_tiles, mt_base + 4 * wt, split, row_base, lane, rs);
}

std::atomic<int> g_units{256};                       // compute units of the device (gemm_set_units): every model on it sets the same value

template <int EPI, int PL, int FMT>
void launch_large_one(const GemmArgs& a, dim3 grid, hipStream_t st) {
  static std::once_flag attr_once;                  // raise the dynamic LDS limit once per instantiation, from any thread
  constexpr int lds = LargeTiling<PL>::LDS_BYTES;
  std::call_once(attr_once, [] {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_large_kernel<EPI, PL, FMT>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  });
  hipLaunchKernelGGL((gemm_large_kernel<EPI, PL, FMT>), grid, dim3(LG_THREADS), lds, st, a);
}

// Only the two-term bf16 format uses this form: with one term per activation (fp16, or bf16 without the split) the
// 128-token skinny form was measured faster (fp16 prefill 73.8 k against 66.6 k tokens/s).
template <int EPI>
void launch_large(const GemmArgs& a, int n_tiles, int grid_y, int rows, hipStream_t st) {
  dim3 grid((n_tiles + LG_TILES - 1) / LG_TILES, grid_y, (rows + 32 * LG_TILES - 1) / (32 * LG_TILES));
  if (a.item_expert) grid.z = 1;                    // grid_y is the length of the item list
  launch_large_one<EPI, 2, DT_BF16>(a, grid, st);
}

template <int MT, int EPI, int PL, int FMT, bool ONCE>
void launch_one_form(const GemmArgs& a, dim3 grid, hipStream_t st) {
  static std::once_flag attr_once;                  // raise the dynamic LDS limit once per instantiation, from any thread
  constexpr int lds = Tiling<MT, PL>::LDS_BYTES;
  std::call_once(attr_once, [] {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_skinny_kernel<MT, EPI, PL, FMT, ONCE>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  });
  hipLaunchKernelGGL((gemm_skinny_kernel<MT, EPI, PL, FMT, ONCE>), grid, dim3(GEMM_THREADS), lds, st, a);
}

// Several token tiles (grid z) share a weight tile only in the store form at 64 tokens per tile (two-group calls) and
// in the 128-token forms; an expert group with more rows than a tile is rare enough to keep the streaming mark.
template <int MT, int EPI, int PL, int FMT>
void launch_one(const GemmArgs& a, dim3 grid, hipStream_t st) {
  constexpr bool shared_tiles_possible = MT == 4 || (MT == 2 && EPI == EPI_STORE);
  if (shared_tiles_possible && grid.z > 1 && a.group_off == nullptr) launch_one_form<MT, EPI, PL, FMT, !shared_tiles_possible>(a, grid, st);
  else launch_one_form<MT, EPI, PL, FMT, true>(a, grid, st);
}

// formats built: bf16 activations as one or two terms, fp16 activations as one term
template <int MT, int EPI>
void launch_fmt(const GemmArgs& a, dim3 grid, const Act& x, hipStream_t st) {
  if (x.dtype == DT_F16) launch_one<MT, EPI, 1, DT_F16>(a, grid, st);
  else if (x.planes == 2) launch_one<MT, EPI, 2, DT_BF16>(a, grid, st);
  else launch_one<MT, EPI, 1, DT_BF16>(a, grid, st);
}

template <int EPI>
void launch_mt(const GemmArgs& a, int n_tiles, int grid_y, int mt, const Act& x, hipStream_t st) {
  if (mt > 4) {
    // more than 128 tokens (per expert), two-term bf16 activations: 256 x 256 tiles where they fill the device at
    // least twice over (a grid of 1.25 workgroups per unit takes as long as one of 2), else the 128-token skinny form
    const long wgs = (long)((n_tiles + LG_TILES - 1) / LG_TILES) * grid_y * ((a.T + 32 * LG_TILES - 1) / (32 * LG_TILES));
    if (wgs >= 2L * g_units.load(std::memory_order_relaxed) && x.planes == 2 && x.dtype == DT_BF16) {
      launch_large<EPI>(a, n_tiles, grid_y, a.T, st);
      return;
    }
    mt = 4;
  }
  const int gx = (n_tiles + GEMM_WAVES - 1) / GEMM_WAVES;
  const int mtiles = (a.T + 31) / 32;
  if (mt == 1) launch_fmt<1, EPI>(a, dim3(gx, grid_y, mtiles), x, st);
  else if (mt == 2) launch_fmt<2, EPI>(a, dim3(gx, grid_y, (mtiles + 1) / 2), x, st);
  else launch_fmt<4, EPI>(a, dim3(gx, grid_y, (mtiles + 3) / 4), x, st);
}

// Expert-grouped decode form (two-term bf16 only; the other formats keep the skinny form).  Tile groups per
// workgroup: three or two, whichever divides the groups of an expert and still leaves two workgroups per compute
// unit (measured at the 30B-A3B shape: gate/up, 12 groups, 155 us with one group per workgroup, 145 with two, 146
// with three; down, 16 groups, 77.7 / 77.0 / 78.8); a grid that cannot fill the device anyway takes two.
template <int J, int EPI>
void launch_expert_one(const GemmArgs& a, dim3 grid, hipStream_t st) {
  static std::once_flag attr_once;
  constexpr int lds = 2 * ExpertTiling<J>::KC * 2 * 1024;
  std::call_once(attr_once, [] {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_expert_kernel<J, EPI, 2, DT_BF16>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  });
  hipLaunchKernelGGL((gemm_expert_kernel<J, EPI, 2, DT_BF16>), grid, dim3(GEMM_THREADS), lds, st, a);
}

int expert_tile_groups(int n_tiles, int n_experts, int n_units) {
  const int groups = (n_tiles + W_GROUP - 1) / W_GROUP;
  for (int j = 3; j >= 2; --j)
    if (groups % j == 0 && (long)(groups / j) * n_experts >= 2L * n_units) return j;
  return groups >= 2 ? 2 : 1;
}

template <int EPI>
bool launch_expert(const GemmArgs& a, int n_tiles, int n_experts, const Act& x, hipStream_t st) {
  if (x.planes != 2 || x.dtype != DT_BF16) return false;
  const int j = expert_tile_groups(n_tiles, n_experts, g_units.load(std::memory_order_relaxed));
  if (j < 2) return false;
  const int groups = (n_tiles + W_GROUP - 1) / W_GROUP;
  const dim3 grid((groups + j - 1) / j, n_experts, (a.T + 31) / 32);
  if (j == 2) launch_expert_one<2, EPI>(a, grid, st);
  else launch_expert_one<3, EPI>(a, grid, st);
  return true;
}

// token tiles per workgroup; 8 selects the large-batch form
int pick_mt(int T) { return T <= 32 ? 1 : (T <= 64 ? 2 : (T <= 128 ? 4 : 8)); }

void fill_x(GemmArgs& a, const Act& x) {
  a.x = x.p; a.x_mtiles = x.mtiles();
  a.x_ss = x.ss; a.x_eps = x.eps;
}

}  // namespace

// Store GEMMs of 65..128 tokens run as two 64-token groups (the weights of these small matrices are read twice,
// the second time from cache): measured faster than one 128-token tile (MoE decode q|k|v 1.03 -> 0.75 ms per step,
// output projection 0.91 -> 0.66, router 0.56 -> 0.44 with the split planning that knows of the two groups; the same
// trick one size down, two 32-token groups for 33..64 tokens, was measured slower).
static int store_mt(int T) { return (T > 64 && T <= 128) ? 2 : pick_mt(T); }
static int store_token_groups(int T) { return (T > 64 && T <= 128) ? 2 : 1; }

int gemm_max_splits() { return 16; }

void gemm_set_units(int n_units) { g_units.store(n_units > 0 ? n_units : 1, std::memory_order_relaxed); }

// Split-K planning.  A compute unit takes in only so many bytes per microsecond however many waves it holds, so
// what counts is that every unit gets the same number of bytes: the grid is kept at or just under one workgroup
// per unit (a grid of 1.2 workgroups per unit takes as long as one of 2), with as few planes as that allows.
static int ksteps_for(int K, int splits) { return (K / 16 + splits - 1) / splits; }

// k-steps that one round of the skinny form's main loop covers (a ring of four weight batches); a K range that is
// not a multiple of it is padded with masked k-steps whose loads are still issued
static int kstep_round(int T, int planes, int dtype) {
  int mt = store_mt(T);
  if (mt > 4) mt = 4;
  const int pl = dtype == DT_F16 ? 1 : planes;
  const int kc = (mt == 1 && pl == 2) ? 12 : ((32 / (mt * pl)) > 16 ? 16 : (32 / (mt * pl)));   // Tiling<MT, PL>::KC
  return 2 * kc;
}

int gemm_plan_splits(int N, int K, int T, int max_splits, int n_units, int planes, int dtype) {
  const int per = GEMM_WAVES;                                          // weight tiles per workgroup
  const int groups = ((N + 31) / 32 + per - 1) / per * store_token_groups(T);   // workgroups per split
  const int KS = K / 16;
  int want = n_units / groups;                      // floor: never more workgroups than units
  if (want > max_splits) want = max_splits;
  if (want > KS / 8) want = KS / 8;                 // at least eight k-steps per split
  if (want < 1) want = 1;
  // A workgroup's time goes with the k-steps its loop runs, padding included, so among the split counts that fit the
  // device the one with the fewest padded k-steps per split wins, and of several such the one with the fewest planes
  // (measured at the 4B shape, 64 tokens: output projection, K = 4096, 12 planes 11.2 us, 8 planes 9.9 us; down
  // projection, K = 9728, 12 planes 17.4 us, 10 planes 16.4 us: both pad 22 and 51 k-steps to 32 and 64).
  const int round = kstep_round(T, planes, dtype);
  int best = 1, best_padded = 0x7FFFFFFF;
  for (int s = 1; s <= want; ++s) {
    const int ksper = ksteps_for(K, s);
    const int padded = (ksper + round - 1) / round * round;
    if (padded < best_padded) { best_padded = padded; best = s; }
  }
  const int ksper = ksteps_for(K, best);
  return (KS + ksper - 1) / ksper;                  // no empty split
}

// Long calls (prefill chunks): a narrow output (the o and down projections) gives the 256 x 256 form too few
// workgroups; two K halves double them, at the price of a second fp32 plane that the consumer adds.
int gemm_plan_splits_long(int N, int T, int planes, int dtype, int n_units) {
  if (planes != 2 || dtype != DT_BF16) return 1;      // the large form is used for two-term bf16 only
  const long wgs = (long)(((N + 31) / 32 + LG_TILES - 1) / LG_TILES) * ((T + 32 * LG_TILES - 1) / (32 * LG_TILES));
  return (wgs < 2L * n_units && 2 * wgs >= 2L * n_units) ? 2 : 1;
}

hipError_t gemm_store(const LinearW& w, const Act& x, int T, float* y, int ldy, int splits, hipStream_t st) {
  GemmArgs a = {};
  fill_x(a, x);
  int tiles = 0;
  for (int i = 0; i < 3; ++i) { a.w[i] = w.seg[i]; a.w_tiles[i] = (w.rows[i] + 31) / 32; tiles += a.w_tiles[i]; }
  a.N = w.N; a.K = w.K; a.T = T;
  a.ksteps_per_split = ksteps_for(w.K, splits);   // same rule as gemm_plan_splits
  a.y = y; a.ldy = ldy;
  launch_mt<EPI_STORE>(a, tiles, splits, store_mt(T), x, st);
  return hipGetLastError();
}

hipError_t gemm_swiglu(const h16_t* w_gate_up, int F, int K, const Act& x, int T, const Act& act, hipStream_t st) {
  GemmArgs a = {};
  fill_x(a, x);
  a.w[0] = w_gate_up; a.w_tiles[0] = F / 16;
  a.N = 2 * F; a.K = K; a.T = T;
  a.ksteps_per_split = K / 16;
  a.act = act.p; a.act_mtiles = act.mtiles();
  launch_mt<EPI_SWIGLU>(a, a.w_tiles[0], 1, pick_mt(T), x, st);
  return hipGetLastError();
}

// Token-tile height of the expert-grouped kernels.  An expert's weights are streamed once per tile of 32 * mt rows
// and every tile reads 32 * mt activation rows whether or not they exist, so the tile should just cover the rows an
// expert is expected to get (decode: a handful; prefill: hundreds); the grid covers max_rows and workgroups past an
// expert's last row exit at once.
static int grouped_mt(int expected_rows) {
  return expected_rows <= 16 ? 1 : (expected_rows <= 40 ? 2 : (expected_rows <= 128 ? 4 : 8));
}

// The item list serves the 256 x 256 form only: two-term bf16 activations, more than 128 expected rows per expert,
// and enough items to fill the device twice (the condition under which launch_mt takes that form).
int gemm_grouped_item_rows(int E, int F, int N, const Act& x, int n_pairs, int expected_rows) {
  if (x.planes != 2 || x.dtype != DT_BF16 || grouped_mt(expected_rows) != 8) return 0;
  const long items = n_pairs / (32 * LG_TILES);     // at least this many full tiles
  const long units = g_units.load(std::memory_order_relaxed);
  const long xg = (F / 16 + LG_TILES - 1) / LG_TILES, xd = ((N + 31) / 32 + LG_TILES - 1) / LG_TILES;
  (void)E;
  return (xg * items >= 2 * units && xd * items >= 2 * units) ? 32 * LG_TILES : 0;
}

hipError_t gemm_grouped_swiglu(const h16_t* w_gate_up, int E, int F, int K, const Act& x, const int32_t* x_rows,
                               const int32_t* group_off, int max_rows, int expected_rows, const Act& act,
                               const GroupItems* items, hipStream_t st) {
  if (x.ss && x_rows) return hipErrorInvalidValue;   // the epilogue would need the row list to find a row's factor
  GemmArgs a = {};
  fill_x(a, x);
  a.x_rows = x_rows;
  a.w[0] = w_gate_up; a.w_tiles[0] = F / 16;
  a.N = 2 * F; a.K = K; a.T = max_rows;
  a.ksteps_per_split = K / 16;
  a.act = act.p; a.act_mtiles = act.mtiles();
  a.group_off = group_off; a.w_expert_stride = packed_weight_elems(2 * F, K);
  if (items) {
    a.item_expert = items->expert; a.item_tile = items->tile;
    launch_large<EPI_SWIGLU>(a, a.w_tiles[0], items->max_items, max_rows, st);
    return hipGetLastError();
  }
  if (grouped_mt(expected_rows) == 1 && launch_expert<EPI_SWIGLU>(a, a.w_tiles[0], E, x, st)) return hipGetLastError();
  launch_mt<EPI_SWIGLU>(a, a.w_tiles[0], E, grouped_mt(expected_rows), x, st);
  return hipGetLastError();
}

hipError_t gemm_grouped_store(const h16_t* w, int E, int N, int K, const Act& x, const int32_t* group_off,
                              int max_rows, int expected_rows, float* y, const GroupItems* items, hipStream_t st) {
  GemmArgs a = {};
  fill_x(a, x);
  a.w[0] = w; a.w_tiles[0] = (N + 31) / 32;
  a.N = N; a.K = K; a.T = max_rows;
  a.ksteps_per_split = K / 16;
  a.y = y; a.ldy = N;
  a.group_off = group_off; a.w_expert_stride = packed_weight_elems(N, K);
  if (items) {
    a.item_expert = items->expert; a.item_tile = items->tile;
    launch_large<EPI_STORE>(a, a.w_tiles[0], items->max_items, max_rows, st);
    return hipGetLastError();
  }
  if (grouped_mt(expected_rows) == 1 && launch_expert<EPI_STORE>(a, a.w_tiles[0], E, x, st)) return hipGetLastError();
  launch_mt<EPI_STORE>(a, a.w_tiles[0], E, grouped_mt(expected_rows), x, st);
  return hipGetLastError();
}

// Routed form of the expert-grouped gate/up GEMM at decode: no grouping pass; every workgroup finds its expert's
// pairs in the routing table (route_idx[token * top_k + slot] = expert), reads the token's row of x and writes act
// in expert order (pairs of expert 0 first, in pair order: what the counting sort produces).  The launch also
// publishes group_off[E + 1] and pair_pos[n_pairs] of that order, which the down GEMM and the combine then read.
bool gemm_routed_form(int E, int F, const Act& x, int n_pairs, int expected_rows) {
  if (x.planes != 2 || x.dtype != DT_BF16 || grouped_mt(expected_rows) != 1) return false;
  if (n_pairs > 16 * GEMM_THREADS) return false;    // at most 16 table entries per thread of a workgroup
  return expert_tile_groups(F / 16, E, g_units.load(std::memory_order_relaxed)) >= 2;
}

hipError_t gemm_routed_swiglu(const h16_t* w_gate_up, int E, int F, int K, const Act& x, const int32_t* route_idx,
                              int n_pairs, int top_k, int max_rows, const Act& act, int32_t* group_off,
                              int32_t* pair_pos, hipStream_t st) {
  GemmArgs a = {};
  fill_x(a, x);
  a.w[0] = w_gate_up; a.w_tiles[0] = F / 16;
  a.N = 2 * F; a.K = K; a.T = max_rows;
  a.ksteps_per_split = K / 16;
  a.act = act.p; a.act_mtiles = act.mtiles();
  a.w_expert_stride = packed_weight_elems(2 * F, K);
  a.route_idx = route_idx; a.n_pairs = n_pairs; a.top_k = top_k;
  a.pub_group_off = group_off; a.pub_pair_pos = pair_pos;
  if (!launch_expert<EPI_SWIGLU>(a, a.w_tiles[0], E, x, st)) return hipErrorInvalidValue;
  return hipGetLastError();
}

int lmhead_tiles(int vocab) { return (vocab + 31) / 32; }

hipError_t gemm_lmhead(const h16_t* w_lm, int V, int K, const Act& x, int T, float* logits, float* part,
                       const uint64_t* seeds, const float* temperature, const int32_t* sample_pos,
                       const int32_t* row_seq, bool draw, hipStream_t st) {
  if (x.ss) return hipErrorInvalidValue;              // the LM-head epilogue takes finished rows only
  GemmArgs a = {};
  fill_x(a, x);
  a.w[0] = w_lm; a.w_tiles[0] = (V + 31) / 32;
  a.N = V; a.K = K; a.T = T;
  a.ksteps_per_split = K / 16;
  a.logits = logits; a.part = part; a.seeds = seeds; a.temperature = temperature; a.sample_pos = sample_pos;
  a.row_seq = row_seq; a.draw = draw ? 1 : 0;
  launch_mt<EPI_LMHEAD>(a, a.w_tiles[0], 1, pick_mt(T), x, st);
  return hipGetLastError();
}

}  // namespace rlx
