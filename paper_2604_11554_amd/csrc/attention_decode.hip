// Decode attention over the paged 16-bit KV pool, load-balanced by key count.
//
// One new token per sequence; the 16 MFMA columns of a tile are the query heads of one KV head
// (group <= 16), so a KV page is read once for all heads of its group.  The work of a step is the
// sequence of 32-key units of all (sequence, KV head) pairs laid end to end; every workgroup takes a
// contiguous share of it, all shares within one unit of each other (the plan is built once per step,
// contexts being the same for every layer), so the grid is exactly resident (two workgroups per compute unit) and every workgroup streams
// for the whole kernel instead of paying its start-up and wind-down latency per 256 keys.  Within a
// share the four waves take units round-robin, each keeping the next unit's pages in flight while it
// works on the current one.  Where a (sequence, KV head) pair lies inside one share its output is
// final; where it straddles shares each part leaves (o, m, l) and a small second kernel merges the
// parts in share order (deterministic).
//
// Shared prompt prefixes (sequences of one sampling group list the same pages for their prompt): the descriptor
// `shared` names, per sequence, how many leading units are served by prefix tiles instead.  A prefix tile is
// (subgroup of up to 32 / group sequences, KV head, chunk of units): the 32 columns of its two MFMA column tiles
// are the query heads of all its member sequences, so the shared pages are read once per subgroup (the eight
// responses of a prompt at the 4B shape) instead of once per sequence; the per-sequence kernel starts after the
// shared units, and the merge kernel adds the prefix parts first.
#include "attn_core.h"

namespace rlx {
namespace {


template <int HD>
struct PageRegs {
  h16x8 k0[HD / 32], k1[HD / 32], vf[HD / 16];
  bool ok0, ok1;
};

// A run: up to 64 consecutive units of one (sequence, KV head) inside this workgroup's share (64 units = one
// register window of the block table).  A segment -- the part of a pair that lies in the share -- is one or
// more runs; the online softmax state lives across the runs of a segment.  All fields are wave-uniform.
// Views into the shared-prefix descriptor (kernels.h); `on` is false when there is none or it was built for
// another batch size, and every index read from it is clamped by its user.
struct SharedView {
  bool on;
  int n_tiles, max_tiles;
  const int32_t *start_unit, *tile0, *n_chunks, *col0, *t_row, *t_kvh, *t_lo, *t_hi, *t_mem;
};
__device__ __forceinline__ SharedView shared_view(const int32_t* sp, int n_seqs, int Hkv) {
  SharedView v = {};
  v.on = sp != nullptr && sp[0] == n_seqs;
  if (!v.on) return v;
  v.max_tiles = shared_prefix_max_tiles(n_seqs, Hkv);
  v.n_tiles = min(max(sp[1], 0), v.max_tiles);
  const int32_t* p = sp + SP_HDR;
  v.start_unit = p; v.tile0 = p + n_seqs; v.n_chunks = p + 2 * n_seqs; v.col0 = p + 3 * n_seqs;
  p += 4 * (size_t)n_seqs;
  v.t_row = p; v.t_kvh = p + v.max_tiles; v.t_lo = p + 2 * (size_t)v.max_tiles; v.t_hi = p + 3 * (size_t)v.max_tiles;
  v.t_mem = p + 4 * (size_t)v.max_tiles;
  return v;
}
// units of sequence `seq` that prefix tiles serve: never all of them (its own kernel keeps at least one unit)
__device__ __forceinline__ int shared_units_of(const SharedView& v, int seq, int ctx) {
  return v.on ? min(max(v.start_unit[seq], 0), ctx / 32) : 0;
}

// Shares of two sizes: workgroups 0 .. H-1 take CA units each, the others CB = CA - 1, which may be zero (plan
// header: CA, total, CB, H).
struct Shares {
  int CA, CB, H, U;
  __device__ __forceinline__ int start(int w) const { return w < H ? w * CA : H * CA + (w - H) * CB; }
  __device__ __forceinline__ int of_unit(int x) const { return x < H * CA ? x / CA : H + (x - H * CA) / max(CB, 1); }
};
__device__ __forceinline__ Shares load_shares(const int32_t* hdr) { return Shares{hdr[0], hdr[2], hdr[3], hdr[1]}; }

struct Run {
  int seq, kvh, ctx, np;     // np: units of the whole pair, counted from unit u0 of the sequence
  int u0;                    // units before this pair's first one (served by prefix tiles)
  int pb, pe;                // units [pb, pe) of the pair are this share's segment
  int lo, hi;                // units [lo, hi) of the pair are this run
  bool seg_start, seg_end, valid;
};

template <int HD, int PL, int FMT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_decode_kernel(AttnDecodeArgs a) {
  constexpr int DT = HD / 16, KS = HD / 32, PS = HD + 4;
  __shared__ f32x4 lds_o[2 * DT * WAVE];
  __shared__ float lds_ml[2 * 2 * WAVE];
  __shared__ u32x4 lds_q[PL * KS * WAVE];            // query fragments of the current segment, MFMA operand order

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c16 = lane & 15, g = lane >> 4;
  const int group = a.Hq / a.Hkv;
  const bool col_ok = c16 < group;
  const int w = blockIdx.x;
  const Shares sh = load_shares(a.plan_hdr);
  const int U = sh.U;
  int u = sh.start(w);
  const int u_end = min(U, sh.start(w + 1));
  if (u >= u_end) return;                            // uniform over the workgroup
  int seq = a.wg_seq[w];
  const float scale = rsqrtf((float)HD);
  const size_t page = (size_t)2 * 16 * HD;

  // ---- run generator: the per-sequence plan entries are held in a 64-lane register window ----
  const SharedView sv = shared_view(a.shared, a.n_seqs, a.Hkv);
  int seq0 = seq;
  int32_t wpre = a.unit_prefix[min(seq0 + lane, a.n_seqs)];
  int32_t wctx = a.ctx_lens[min(seq0 + lane, a.n_seqs - 1)];
  int32_t wst = shared_units_of(sv, min(seq0 + lane, a.n_seqs - 1), wctx);
  int rem_lo = 0, rem_hi = 0;                        // rest of the current segment
  Run seg = {};
  auto next_run = [&](Run& r) {
    if (rem_lo < rem_hi) {                           // the segment continues in another table window
      r = seg;
      r.lo = rem_lo; r.hi = min(rem_hi, rem_lo + 64);
      r.seg_start = false; r.seg_end = r.hi == rem_hi;
      rem_lo = r.hi;
      return;
    }
    r.valid = false;
    while (u < u_end && seq < a.n_seqs) {
      if (seq - seq0 > 62) {                         // slide the window (rare: 63 sequences inside one share)
        seq0 = seq;
        wpre = a.unit_prefix[min(seq0 + lane, a.n_seqs)];
        wctx = a.ctx_lens[min(seq0 + lane, a.n_seqs - 1)];
        wst = shared_units_of(sv, min(seq0 + lane, a.n_seqs - 1), wctx);
      }
      const int p0 = __builtin_amdgcn_readlane(wpre, seq - seq0);
      const int np = __builtin_amdgcn_readlane(wpre, seq - seq0 + 1) - p0;
      if (np == 0) { ++seq; continue; }              // inert sequence: no units
      const int base = a.Hkv * p0;
      const int kvh = (u - base) / np;
      if (kvh >= a.Hkv) return;                      // inconsistent plan: stop rather than index past the pool
      const int xs = base + kvh * np;                // first unit of this (sequence, KV head)
      seg.seq = seq; seg.kvh = kvh; seg.np = np;
      seg.ctx = __builtin_amdgcn_readlane(wctx, seq - seq0);
      seg.u0 = __builtin_amdgcn_readlane(wst, seq - seq0);
      seg.pb = u - xs; seg.pe = min(np, u_end - xs);
      seg.valid = true;
      r = seg;
      r.lo = seg.pb; r.hi = min(seg.pe, seg.pb + 64);
      r.seg_start = true; r.seg_end = r.hi == seg.pe;
      rem_lo = r.hi; rem_hi = seg.pe;
      u = xs + seg.pe;
      if (seg.pe == np && kvh == a.Hkv - 1) ++seq;
      return;
    }
  };
  // block-table window of a run: lane holds the entries of blocks 2 (u0 + lo) + lane and + 64
  auto load_window = [&](const Run& r, int32_t& t0, int32_t& t1) {
    const int32_t* table = a.block_table + (size_t)r.seq * a.max_blocks;
    const int jb = 2 * (r.u0 + r.lo) + lane;
    const int j0 = min(jb, a.max_blocks - 1), j1 = min(jb + 64, a.max_blocks - 1);
    t0 = table[j0]; t1 = table[j1];                  // unconditional, clamped; masked below
    if (jb >= a.max_blocks) t0 = -1;
    if (jb + 64 >= a.max_blocks) t1 = -1;
  };
  // The waves share the fetch of a segment's query fragments; they stay in LDS (registers hold two units of pages).
  // The fragments of the next run's pair are requested a whole run ahead (the run generator looks one run ahead
  // anyway) and only written to LDS at the switch, so that a new segment does not begin with a round trip.
  constexpr int QPW = (PL * KS + 3) / 4;             // fragments fetched by each wave
  auto fetch_queries = [&](const Run& r, u32x4 (&q)[QPW]) {
    const int head = r.kvh * group + (col_ok ? c16 : 0);
#pragma unroll
    for (int i = 0; i < QPW; ++i) {
      const int f = min(wave + 4 * i, PL * KS - 1);  // a slot without a fragment repeats the last one; never written
      const int p = f / KS, ks = f % KS;
      q[i] = *reinterpret_cast<const u32x4*>(a.q.p + p * a.q.plane + ((size_t)r.seq * a.Hq + head) * HD + 32 * ks + 8 * g);
    }
  };
  auto put_queries = [&](const u32x4 (&q)[QPW]) {
    const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < QPW; ++i)
      if (wave + 4 * i < PL * KS) lds_q[(wave + 4 * i) * WAVE + lane] = col_ok ? q[i] : z;
  };
  auto qf = [&](int p, int, int ks) { return __builtin_bit_cast(h16x8, lds_q[(p * KS + ks) * WAVE + lane]); };

  Run cur, nxt;
  next_run(cur);
  if (!cur.valid) return;
  int32_t tb0, tb1, tbn0, tbn1;
  load_window(cur, tb0, tb1);
  u32x4 qpre[QPW];
  fetch_queries(cur, qpre);
  put_queries(qpre);
  __syncthreads();

  // Page loads of unit i of run r (table window t0/t1).  They are unconditional: a slot with no unit behind it
  // (`live` false, i clamped into the run) reads one fixed row of the pool with every lane, which costs cache
  // hits and no memory traffic.
  auto issue = [&](const Run& r, int32_t t0, int32_t t1, int i, bool live, PageRegs<HD>& pr) {
    const int rel = 2 * (i - r.lo);                  // uniform, 0 .. 126
    const int32_t sel = rel < 64 ? t0 : t1;
    int64_t b0 = __builtin_amdgcn_readlane(sel, rel & 63);
    int64_t b1 = __builtin_amdgcn_readlane(sel, (rel + 1) & 63);
    const bool has1 = (2 * (r.u0 + i) + 1) * 16 < r.ctx + 1;
    pr.ok0 = live && b0 >= 0 && b0 < a.n_blocks;
    pr.ok1 = live && has1 && b1 >= 0 && b1 < a.n_blocks;
    if (!pr.ok0) b0 = 0;                             // keep the loads in bounds; scores are masked
    if (!pr.ok1) b1 = b0;
    const h16_t* kp0 = a.pool_layer + ((size_t)b0 * a.Hkv + r.kvh) * page;
    const h16_t* kp1 = a.pool_layer + ((size_t)b1 * a.Hkv + r.kvh) * page;
    const h16_t* vp0 = kp0 + 16 * HD;
    const h16_t* vp1 = kp1 + 16 * HD;
    const int koff0 = pr.ok0 ? c16 * HD + 8 * g : 0, koff1 = pr.ok1 ? c16 * HD + 8 * g : 0;
    const int voff0 = pr.ok0 ? c16 * 16 + 4 * g : 0, voff1 = pr.ok1 ? c16 * 16 + 4 * g : 0;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      pr.k0[ks] = load_stream_16(kp0 + koff0 + 32 * ks);
      pr.k1[ks] = load_stream_16(kp1 + koff1 + 32 * ks);
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
      pr.vf[dt] = load_2x4_stream(vp0 + 256 * dt + voff0, vp1 + 256 * dt + voff1);
  };

  WaveState<HD, 1> st;
  PageRegs<HD> ra, rb;
  issue(cur, tb0, tb1, min(cur.lo + wave, cur.hi - 1), cur.lo + wave < cur.hi, ra);
  bool first_seg = true;

  for (;;) {                                         // one run per iteration; uniform
    next_run(nxt);
    const bool more = nxt.valid;
    if (!more) nxt = cur;                            // keeps the look-ahead loads below in bounds
    load_window(nxt, tbn0, tbn1);
    fetch_queries(nxt, qpre);                        // unconditional, like every load of this loop
    if (cur.seg_start) st.reset();
    const int key_end = cur.ctx + 1;
    const int pos_col[1] = {cur.ctx};
    auto step = [&](int i, const PageRegs<HD>& pr, bool valid) {
      pair_step<HD, 1, PL, FMT>(st, pr.k0, pr.k1, pr.vf, qf, 32 * (cur.u0 + i), 32 * (cur.u0 + i) + 16, pr.ok0 && valid,
                                pr.ok1 && valid, key_end, pos_col, scale, g);
    };

    // Two register sets alternate: while one unit is multiplied the next one's pages are in flight.  The loop
    // body has no branch around a load (a unit index past the wave's last one is clamped and its step masked),
    // so the hardware counters let each step wait for its own pages only.  The slot after the wave's last unit
    // fetches its first unit of the next run, so the stream does not drain between runs.
    const int first = cur.lo + wave;
    const int n_my = first < cur.hi ? (cur.hi - first + 3) / 4 : 0;
    const int last = first + 4 * (n_my - 1);
    const int nfirst = min(nxt.lo + wave, nxt.hi - 1);
    const bool nlive = more && nxt.lo + wave < nxt.hi;
    for (int k = 0; k < n_my; k += 2) {
      const int i = first + 4 * k;
      issue(cur, tb0, tb1, min(i + 4, last), i + 4 <= last, rb);
      asm volatile("" ::: "memory");                 // query fragments are re-read from LDS, not kept in registers
      __builtin_amdgcn_sched_barrier(0);             // the next unit's loads go out before this unit's math
      step(i, ra, true);
      {
        const bool beyond = i + 8 > last;
        Run rs = cur;
        if (beyond) rs = nxt;
        issue(rs, beyond ? tbn0 : tb0, beyond ? tbn1 : tb1, beyond ? nfirst : i + 8, !beyond || nlive, ra);
      }
      asm volatile("" ::: "memory");
      __builtin_amdgcn_sched_barrier(0);
      step(i + 4, rb, k + 1 < n_my);
    }
    if (n_my == 0) issue(nxt, tbn0, tbn1, nfirst, nlive, ra);   // this wave had no unit in the run

    if (cur.seg_end) {
      st.finish_denominators();
      merge_waves<HD, 1>(st, lds_o, lds_ml, wave, lane);
      if (wave == 0 && col_ok) {
        const int head = cur.kvh * group + c16;
        const bool whole = cur.pb == 0 && cur.pe == cur.np;
        if (whole && cur.u0 == 0) {
          store_column<HD, 1, PL, FMT>(st, 0, a.o, cur.seq, head, g);
        } else {                                     // lane holds column c16, rows d = 16 dt + 4 g + {0..3}
          float* dst = whole ? a.seq_part + (((size_t)cur.seq * a.Hkv + cur.kvh) * group + c16) * PS
                             : a.part + ((size_t)(w * 2 + (first_seg ? 0 : 1)) * group + c16) * PS;
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) *reinterpret_cast<f32x4*>(dst + 16 * dt + 4 * g) = st.o[0][dt];
          if (g == 0) { dst[HD] = st.m[0]; dst[HD + 1] = st.l[0]; }
        }
      }
      first_seg = false;
    }
    if (!more) break;
    if (nxt.seg_start) put_queries(qpre);            // every wave is past the merge: the old fragments are dead
    __syncthreads();                                 // new fragments visible; wave 0 is done with the merge buffers
    cur = nxt; tb0 = tbn0; tb1 = tbn1;
  }
}

// Prefix tiles: workgroup t, t + grid, ... takes tile t of the descriptor.  The NCT x 16 columns are (member, head of
// the KV head's group); every key of the tile's units is visible to every member (the pages are full and shared).
// The four waves take units round-robin and are merged through LDS; (o, m, l) of all columns go to pre_part.  The
// query fragments of a tile sit in LDS (with two column tiles they would take half the register file).
template <int HD, int PL, int FMT, int NCT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_decode_prefix_kernel(AttnDecodeArgs a) {
  constexpr int DT = HD / 16, KS = HD / 32, PS = HD + 4, NQ = PL * NCT * KS;
  __shared__ f32x4 lds_o[2 * NCT * DT * WAVE];
  __shared__ float lds_ml[2 * NCT * 2 * WAVE];
  __shared__ u32x4 lds_q[NQ * WAVE];                 // fragment (p, c, ks) at ((p * NCT + c) * KS + ks) * 64 + lane
  const SharedView sv = shared_view(a.shared, a.n_seqs, a.Hkv);
  if (!sv.on) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c16 = lane & 15, g = lane >> 4;
  const int group = a.Hq / a.Hkv;
  const float scale = rsqrtf((float)HD);
  const size_t page = (size_t)2 * 16 * HD;
  for (int t = blockIdx.x; t < sv.n_tiles; t += gridDim.x) {
    const int row = min(max(sv.t_row[t], 0), a.n_seqs - 1);
    const int kvh = min(max(sv.t_kvh[t], 0), a.Hkv - 1);
    const int lo = max(sv.t_lo[t], 0), hi = min(sv.t_hi[t], a.max_blocks / 2);
    // the waves share the fetch of the tile's query fragments
#pragma unroll
    for (int i = 0; i < (NQ + 3) / 4; ++i) {
      const int f = wave + 4 * i;
      if (f < NQ) {
        const int p = f / (NCT * KS), c = (f / KS) % NCT, ks = f % KS;
        const int col = 16 * c + c16, mi = col / group;
        const int mem = mi < 16 ? sv.t_mem[(size_t)t * 16 + mi] : -1;
        const bool col_ok = mem >= 0 && mem < a.n_seqs;
        const int head = kvh * group + col % group;
        const u32x4 z = {0u, 0u, 0u, 0u};
        u32x4 q = z;
        if (col_ok)
          q = *reinterpret_cast<const u32x4*>(a.q.p + p * a.q.plane + ((size_t)mem * a.Hq + head) * HD + 32 * ks + 8 * g);
        lds_q[f * WAVE + lane] = q;
      }
    }
    __syncthreads();
    auto qf = [&](int p, int c, int ks) {
      return __builtin_bit_cast(h16x8, lds_q[((p * NCT + c) * KS + ks) * WAVE + lane]);
    };
    WaveState<HD, NCT> st;
    st.reset();
    const int32_t* table = a.block_table + (size_t)row * a.max_blocks;
    int pos_col[NCT];
#pragma unroll
    for (int c = 0; c < NCT; ++c) pos_col[c] = 0x7FFFFFFF;
    for (int i = lo + wave; i < hi; i += 4) {          // 2 i + 1 < max_blocks by the clamp of hi
      int64_t b0 = table[2 * i], b1 = table[2 * i + 1];
      const bool ok0 = b0 >= 0 && b0 < a.n_blocks, ok1 = b1 >= 0 && b1 < a.n_blocks;
      if (!ok0) b0 = 0;                                // keep the loads in bounds; scores are masked
      if (!ok1) b1 = b0;
      const h16_t* kp0 = a.pool_layer + ((size_t)b0 * a.Hkv + kvh) * page;
      const h16_t* kp1 = a.pool_layer + ((size_t)b1 * a.Hkv + kvh) * page;
      h16x8 k0[KS], k1[KS], vf[DT];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        k0[ks] = load_h16x8(kp0 + c16 * HD + 32 * ks + 8 * g);     // the tiles of a group read these pages again:
        k1[ks] = load_h16x8(kp1 + c16 * HD + 32 * ks + 8 * g);     // ordinary loads (the streaming mark cost 25 % here)
      }
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
        vf[dt] = load_2x4(kp0 + 16 * HD + (size_t)(16 * dt + c16) * 16 + 4 * g,
                          kp1 + 16 * HD + (size_t)(16 * dt + c16) * 16 + 4 * g);
      asm volatile("" ::: "memory");                   // query fragments are re-read from LDS, not kept in registers
      pair_step<HD, NCT, PL, FMT>(st, k0, k1, vf, qf, 32 * i, 32 * i + 16, ok0, ok1, 0x7FFFFFFF, pos_col, scale, g);
    }
    st.finish_denominators();
    merge_waves<HD, NCT>(st, lds_o, lds_ml, wave, lane);
    if (wave == 0) {
#pragma unroll
      for (int c = 0; c < NCT; ++c) {
        float* dst = a.pre_part + ((size_t)t * SP_COLS + 16 * c + c16) * PS;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) *reinterpret_cast<f32x4*>(dst + 16 * dt + 4 * g) = st.o[c][dt];
        if (g == 0) { dst[HD] = st.m[c]; dst[HD + 1] = st.l[c]; }
      }
    }
    __syncthreads();                                   // the merge buffers and the fragments are free for the next tile
  }
}

// One 64-thread workgroup per (sequence, KV head): inert rows are zeroed; a pair that one share covered and no
// prefix precedes is already final; otherwise the parts are merged in a fixed order: prefix chunks in key order,
// then the pair's own part (one share) or parts (share order).
template <int HD>
__global__ __launch_bounds__(256) void attn_decode_merge_kernel(AttnDecodeArgs a) {
  constexpr int PS = HD + 4;
  const int seq = blockIdx.x / a.Hkv, kvh = blockIdx.x % a.Hkv;
  const int lane = threadIdx.x;
  const int group = a.Hq / a.Hkv, PL = a.o.planes, mtiles = a.o.mtiles();
  const int np = a.unit_prefix[seq + 1] - a.unit_prefix[seq];
  const Shares sh = load_shares(a.plan_hdr);
  const int xs = a.Hkv * a.unit_prefix[seq] + kvh * np;
  const int w_first = np ? sh.of_unit(xs) : 0, w_last = np ? sh.of_unit(xs + np - 1) : 0;
  const SharedView sv = shared_view(a.shared, a.n_seqs, a.Hkv);
  const int su = np ? shared_units_of(sv, seq, a.ctx_lens[seq]) : 0;
  if (np && w_first == w_last && su == 0) return;
  int n_chunks = 0, tile0 = 0, col0 = 0;
  if (su > 0) {
    n_chunks = min(max(sv.n_chunks[seq], 0), SP_MAX_CHUNKS);
    tile0 = max(sv.tile0[seq], 0);
    col0 = min(max(sv.col0[seq], 0), SP_COLS - group);
  }
  for (int uu = lane; uu < group * HD / 8; uu += (int)blockDim.x) {   // one pass: the block has a thread per slice
    const int j = uu / (HD / 8), d0 = (uu % (HD / 8)) * 8;
    float m = -INFINITY, l = 0.f;
    float o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = 0.f;
    auto add = [&](const f32x4& va, const f32x4& vb, float ms, float ls) {
      if (ms == -INFINITY) return;
      const float mn = fmaxf(m, ms);
      const float aa = (m == -INFINITY) ? 0.f : __expf(m - mn);
      const float ab = __expf(ms - mn);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        o[e] = o[e] * aa + va[e] * ab;
        o[4 + e] = o[4 + e] * aa + vb[e] * ab;
      }
      l = l * aa + ls * ab;
      m = mn;
    };
    auto add_at = [&](const float* p) {
      add(*reinterpret_cast<const f32x4*>(p + d0), *reinterpret_cast<const f32x4*>(p + d0 + 4), p[HD], p[HD + 1]);
    };
    for (int c = 0; c < n_chunks; ++c) {
      const int t = min(tile0 + c * a.Hkv + kvh, sv.max_tiles - 1);
      add_at(a.pre_part + ((size_t)t * SP_COLS + col0 + j) * PS);
    }
    if (np && w_first == w_last) {
      add_at(a.seq_part + (((size_t)seq * a.Hkv + kvh) * group + j) * PS);
    } else if (np) {
      for (int w0 = w_first; w0 <= w_last; w0 += 4) {
        f32x4 va[4], vb[4];
        float ms[4], ls[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {                // loads first (clamped), merges after
          const int wc = w0 + q <= w_last ? w0 + q : w_last;
          const int slot = xs <= sh.start(wc) ? 0 : 1;   // first segment of its share or not
          const float* p = a.part + ((size_t)(wc * 2 + slot) * group + j) * PS;
          va[q] = *reinterpret_cast<const f32x4*>(p + d0);
          vb[q] = *reinterpret_cast<const f32x4*>(p + d0 + 4);
          ms[q] = p[HD]; ls[q] = p[HD + 1];
        }
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (w0 + q <= w_last) add(va[q], vb[q], ms[q], ls[q]);
      }
    }
    h16_t hi[8], lo[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) split_h16(l > 0.f ? o[e] / l : 0.f, hi[e], lo[e], a.o.dtype);
    h16_t* dst = a.o.p + frag_act_offset(seq, (kvh * group + j) * HD + d0, 0, mtiles, PL);
    u32x4 pk = {(uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16),
                (uint32_t)hi[4] | ((uint32_t)hi[5] << 16), (uint32_t)hi[6] | ((uint32_t)hi[7] << 16)};
    *reinterpret_cast<u32x4*>(dst) = pk;
    if (PL == 2) {
      u32x4 pk2 = {(uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16),
                   (uint32_t)lo[4] | ((uint32_t)lo[5] << 16), (uint32_t)lo[6] | ((uint32_t)lo[7] << 16)};
      *reinterpret_cast<u32x4*>(dst + 512) = pk2;
    }
  }
}

// One workgroup: exclusive prefix of the per-sequence unit counts, the two share sizes, and the sequence in which
// each share starts.
__global__ __launch_bounds__(1024) void attn_plan_kernel(int n_seqs, const int32_t* ctx, const uint8_t* live, int Hkv,
                                                          int n_wgs, const int32_t* shared, int32_t* unit_prefix,
                                                          int32_t* wg_seq, int32_t* hdr) {
  __shared__ int sh[1024];
  __shared__ int carry;
  const int tid = threadIdx.x;
  const SharedView sv = shared_view(shared, n_seqs, Hkv);
  if (tid == 0) carry = 0;
  __syncthreads();
  for (int base = 0; base < n_seqs; base += 1024) {
    const int i = base + tid;
    // units of the sequence's own pairs: those after the ones that prefix tiles serve
    const int v = (i < n_seqs && live[i]) ? (ctx[i] + 1 + 31) / 32 - shared_units_of(sv, i, ctx[i]) : 0;
    sh[tid] = v;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
      const int t = tid >= o ? sh[tid - o] : 0;
      __syncthreads();
      sh[tid] += t;
      __syncthreads();
    }
    if (i < n_seqs) unit_prefix[i] = carry + sh[tid] - v;
    __syncthreads();
    if (tid == 1023) carry += sh[1023];
    __syncthreads();
  }
  const int per_head = carry;
  if (tid == 0) unit_prefix[n_seqs] = per_head;
  __syncthreads();                                   // the prefix is read back below
  const int total = per_head * Hkv;
  // share sizes differ by at most one unit: the units of the step are dealt out evenly and the first H workgroups
  // take the remainder, one unit each.  (One size for all, rounded up, left a tenth of the workgroups without work
  // at the benchmark's contexts; sizes in multiples of four units, so that the four waves of a share get equal
  // counts, made the longer shares up to a tenth longer than the mean, and the waves' counts are unequal anyway
  // wherever a pair's boundary falls inside a share.)  With as many (sequence, KV head) pairs as workgroups and
  // equal contexts a share is exactly a pair: nothing straddles and nothing is left to merge.
  const int q = total / n_wgs, H = total % n_wgs;
  const int CA = q + 1, CB = q;
  if (tid == 0) { hdr[0] = CA; hdr[1] = total; hdr[2] = CB; hdr[3] = H; }
  const Shares shr = Shares{CA, CB, H, total};
  for (int w = tid; w < n_wgs; w += 1024) {
    const int u0 = shr.start(w);
    int lo = 0, hi = n_seqs - 1;                     // largest s with Hkv * prefix[s] <= u0
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (Hkv * unit_prefix[mid] <= u0) lo = mid; else hi = mid - 1;
    }
    wg_seq[w] = u0 < total ? lo : n_seqs;
  }
}

}  // namespace

hipError_t attention_decode_plan(int n_seqs, const int32_t* ctx_lens, const uint8_t* tok_live, int Hkv, int n_wgs,
                                 const int32_t* shared, int32_t* unit_prefix, int32_t* wg_seq, int32_t* hdr,
                                 hipStream_t st) {
  hipLaunchKernelGGL(attn_plan_kernel, dim3(1), dim3(1024), 0, st, n_seqs, ctx_lens, tok_live, Hkv, n_wgs, shared,
                     unit_prefix, wg_seq, hdr);
  return hipGetLastError();
}

// Host side of the descriptor.  A group is a run of consecutive sequences with the same leader (the first of them);
// its shared units are the smallest shared page count of its members, halved.  Groups of one, groups that share
// less than one unit, and models whose 32 columns hold a single sequence get no tiles.
void shared_prefix_build(int n_seqs, int Hq, int Hkv, const int32_t* leader, const int32_t* shared_pages, int32_t* words) {
  const int group = Hq / Hkv, MS = shared_prefix_members(group);
  const int max_tiles = shared_prefix_max_tiles(n_seqs, Hkv);
  const size_t n_words = shared_prefix_words(n_seqs, Hkv);
  for (size_t i = 0; i < n_words; ++i) words[i] = 0;
  int32_t* start_unit = words + SP_HDR;
  int32_t *tile0 = start_unit + n_seqs, *n_chunks = tile0 + n_seqs, *col0 = n_chunks + n_seqs;
  int32_t* t_row = col0 + n_seqs;
  int32_t *t_kvh = t_row + max_tiles, *t_lo = t_kvh + max_tiles, *t_hi = t_lo + max_tiles, *t_mem = t_hi + max_tiles;
  for (int i = 0; i < max_tiles * 16; ++i) t_mem[i] = -1;
  words[0] = n_seqs; words[2] = MS;
  int n_tiles = 0;
  if (MS >= 2) {
    // first pass: groups and their subgroup count, to size the chunks so that the tiles fit
    int n_sub_total = 0;
    for (int b = 0; b < n_seqs;) {
      int e = b + 1;
      while (e < n_seqs && leader[e] == b && leader[b] == b) ++e;
      int units = 0x7FFFFFFF;
      for (int i = b; i < e; ++i) units = shared_pages[i] / 2 < units ? shared_pages[i] / 2 : units;
      if (e - b >= 2 && units > 0) n_sub_total += (e - b + MS - 1) / MS;
      b = e;
    }
    int chunks_cap = n_sub_total ? max_tiles / (n_sub_total * Hkv) : 0;
    if (chunks_cap > SP_MAX_CHUNKS) chunks_cap = SP_MAX_CHUNKS;
    for (int b = 0; b < n_seqs && chunks_cap >= 1;) {
      int e = b + 1;
      while (e < n_seqs && leader[e] == b && leader[b] == b) ++e;
      int units = 0x7FFFFFFF;
      for (int i = b; i < e; ++i) units = shared_pages[i] / 2 < units ? shared_pages[i] / 2 : units;
      if (e - b >= 2 && units > 0) {
        int nc = (units + 7) / 8;                      // at least eight units (256 keys) per chunk
        if (nc > chunks_cap) nc = chunks_cap;
        const int per = (units + nc - 1) / nc;
        nc = (units + per - 1) / per;                  // no empty chunk
        for (int sb = b; sb < e; sb += MS) {
          const int se = sb + MS < e ? sb + MS : e;
          for (int i = sb; i < se; ++i) {
            start_unit[i] = units; tile0[i] = n_tiles; n_chunks[i] = nc; col0[i] = (i - sb) * group;
          }
          for (int c = 0; c < nc; ++c)
            for (int h = 0; h < Hkv; ++h) {
              const int t = n_tiles + c * Hkv + h;
              t_row[t] = b; t_kvh[t] = h; t_lo[t] = c * per; t_hi[t] = (c + 1) * per < units ? (c + 1) * per : units;
              for (int i = sb; i < se; ++i) t_mem[t * 16 + (i - sb)] = i;
            }
          n_tiles += nc * Hkv;
        }
      }
      b = e;
    }
  }
  words[1] = n_tiles;
}

template <int HD, int PL, int FMT>
static void launch_prefix(const AttnDecodeArgs& a, dim3 grid, hipStream_t st) {
  // one column tile holds all members when there is one query head per KV head; two otherwise
  if (shared_prefix_members(a.Hq / a.Hkv) * (a.Hq / a.Hkv) <= 16)
    hipLaunchKernelGGL((attn_decode_prefix_kernel<HD, PL, FMT, 1>), grid, dim3(256), 0, st, a);
  else
    hipLaunchKernelGGL((attn_decode_prefix_kernel<HD, PL, FMT, 2>), grid, dim3(256), 0, st, a);
}

hipError_t attention_decode_prefix(const AttnDecodeArgs& a, hipStream_t st) {
  if (!a.shared) return hipSuccess;
  dim3 grid(a.n_prefix_wgs);
  const bool two = a.q.planes == 2;
  if (a.o.dtype == DT_F16) {
    if (a.hd == 128) launch_prefix<128, 1, DT_F16>(a, grid, st);
    else launch_prefix<64, 1, DT_F16>(a, grid, st);
  } else if (a.hd == 128) {
    if (two) launch_prefix<128, 2, DT_BF16>(a, grid, st);
    else launch_prefix<128, 1, DT_BF16>(a, grid, st);
  } else {
    if (two) launch_prefix<64, 2, DT_BF16>(a, grid, st);
    else launch_prefix<64, 1, DT_BF16>(a, grid, st);
  }
  return hipGetLastError();
}

hipError_t attention_decode(const AttnDecodeArgs& a, hipStream_t st) {
  dim3 grid(a.n_wgs);
  const bool two = a.q.planes == 2;
  // formats built: bf16 with one or two terms, fp16 with one term (checked when the model is created)
  if (a.o.dtype == DT_F16) {
    if (a.hd == 128) hipLaunchKernelGGL((attn_decode_kernel<128, 1, DT_F16>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((attn_decode_kernel<64, 1, DT_F16>), grid, dim3(256), 0, st, a);
  } else if (a.hd == 128) {
    if (two) hipLaunchKernelGGL((attn_decode_kernel<128, 2, DT_BF16>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((attn_decode_kernel<128, 1, DT_BF16>), grid, dim3(256), 0, st, a);
  } else {
    if (two) hipLaunchKernelGGL((attn_decode_kernel<64, 2, DT_BF16>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((attn_decode_kernel<64, 1, DT_BF16>), grid, dim3(256), 0, st, a);
  }
  return hipGetLastError();
}

hipError_t attention_decode_merge(const AttnDecodeArgs& a, hipStream_t st) {
  dim3 grid(a.n_seqs * a.Hkv);
  const int slices = (a.Hq / a.Hkv) * a.hd / 8;      // 8-feature slices of a pair's heads: at most 16 * 128 / 8 = 256
  dim3 block((slices + 63) / 64 * 64);
  if (a.hd == 128) hipLaunchKernelGGL((attn_decode_merge_kernel<128>), grid, block, 0, st, a);
  else hipLaunchKernelGGL((attn_decode_merge_kernel<64>), grid, block, 0, st, a);
  return hipGetLastError();
}

}  // namespace rlx
