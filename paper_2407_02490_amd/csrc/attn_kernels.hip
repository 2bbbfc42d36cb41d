// Causal sparse attention kernels for gfx950 (MI355X).
//
// What is computed: Eq. 1 of the paper, A(M) = softmax(QK^T/sqrt(d) - c(1-M)) V
// with c -> infinity, for the A-shape, Block-Sparse (App. C.4.1) and
// Vertical-Slash (App. C.4.2, Alg. 5) masks, with the online-softmax recurrence
// of Alg. 5 (running max m, running sum l, rescale by exp(m - m_new)).
//
// How (differs from the paper's A100/Triton design on purpose):
//  * One 64-lane wavefront owns one 64-row query block.  Q lives in registers
//    as MFMA B-operand fragments for the whole kernel, O^T is accumulated in
//    registers.
//  * Per 64-key tile the wave computes S^T = K Q^T with v_mfma_f32_32x32x16_bf16
//    (keys on the M axis).  The accumulator layout of S^T is exactly the
//    B-operand layout the second contraction O^T += V^T P^T needs, so P never
//    leaves registers: no LDS round trip, no cross-lane shuffles for P.  The
//    only cross-lane traffic of the softmax is one swap between lanes l and
//    l^32 per 32 query rows for the row max.
//  * K tiles sit in LDS row-major (padded rows); V tiles are transposed on the
//    way in (registers -> LDS as V^T with keys contiguous), so both MFMA A
//    operands are single 16-byte LDS reads.
//  * Tiles are fetched by key index, so a gathered tile of 64 vertical columns
//    costs the same as a contiguous one.  No mask tensor exists anywhere: the
//    element mask is evaluated from (query row, key id) in registers, and only
//    on tiles that can contain a masked element.
//  * A-shape / dense: a workgroup is 4 waves = 4 consecutive query blocks of
//    one head; its K/V tiles are staged once in LDS (double buffered) and
//    shared by the 4 waves.  Block-Sparse / Vertical-Slash: tile lists differ
//    per query block, so a workgroup is a single wave with a private LDS tile
//    and 4 workgroups share a CU.
#include "mfma_tile.h"

namespace minf {

// ---- per-wave setup / epilogue ---------------------------------------------
__device__ inline void wave_init(WaveState &st, const bf16_t *qh, int64_t q_st, int q0, int lane) {
  const int n = lane & 31, h = lane >> 5;
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    const bf16_t *row = qh + (int64_t)(q0 + 32 * nb + n) * q_st + 8 * h;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) st.q[nb][ks] = *reinterpret_cast<const bf16x8 *>(row + 16 * ks);
    st.m[nb] = -INFINITY;
    st.l[nb] = 0.f;
  }
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.o[db][nb][r] = 0.f;
}

// Normalise, convert to bf16, transpose through this wave's LDS region
// (>= 64 * K_PITCH elements) and write O rows with 16-byte coalesced stores.
__device__ inline void wave_finish(WaveState &st, bf16_t *oh, int64_t o_st, int q0, bf16_t *lds,
                                   int lane) {
  const int n = lane & 31, h = lane >> 5;
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    float l = st.l[nb] + __shfl_xor(st.l[nb], 32);
    float inv = l > 0.f ? 1.0f / l : 0.f;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        // registers 4g..4g+3 hold d = 32db + 8g + 4h + (0..3) of query 32nb + n
        f32x2 a = {st.o[db][nb][4 * g + 0] * inv, st.o[db][nb][4 * g + 1] * inv};
        f32x2 b = {st.o[db][nb][4 * g + 2] * inv, st.o[db][nb][4 * g + 3] * inv};
        bf16x2 pa = __builtin_convertvector(a, bf16x2);
        bf16x2 pb = __builtin_convertvector(b, bf16x2);
        uint2 w;
        w.x = *reinterpret_cast<unsigned *>(&pa);
        w.y = *reinterpret_cast<unsigned *>(&pb);
        *reinterpret_cast<uint2 *>(lds + (32 * nb + n) * K_PITCH + 32 * db + 8 * g + 4 * h) = w;
      }
  }
  // LDS operations of one wave execute in issue order; the fences only keep the
  // compiler from moving the reads below above the writes of other lanes.
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    int c = lane + 64 * i;
    int row = c >> 4, col = c & 15;
    uint4 w = *reinterpret_cast<const uint4 *>(lds + row * K_PITCH + col * 8);
    *reinterpret_cast<uint4 *>(oh + (int64_t)(q0 + row) * o_st + col * 8) = w;
  }
}

// ---- one 64 x 64 tile: S^T = K Q^T, mask, online softmax, O^T += V^T P^T ----
// MODE 0: no element is masked.  MODE 1: contiguous keys kbase + idx, mask mp.
// MODE 2: gathered keys cols[idx] (LDS), attended iff key <= query row.
template <int MODE>
__device__ inline void tile_compute(WaveState &st, const bf16_t *ldsK, const bf16_t *ldsVt, int kbase,
                                    const int *cols, const MaskP &mp, float c_log2, int lane) {
  const int n = lane & 31, h = lane >> 5;
  const int prow = perm_row(n);
  f32x16 s[2][2];
#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[mb][nb][r] = 0.f;

#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
      bf16x8 a = *reinterpret_cast<const bf16x8 *>(ldsK + (32 * mb + prow) * K_PITCH + 16 * ks + 8 * h);
      s[mb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, st.q[0][ks], s[mb][0], 0, 0, 0);
      s[mb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, st.q[1][ks], s[mb][1], 0, 0, 0);
    }
  }

  // register r of s[mb][nb] holds key index 32mb + 16(r/8) + 8h + (r%8), query 32nb + n
  if (MODE != 0) {
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
      int keys[16];
      if (MODE == 2) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          int4 a = *reinterpret_cast<const int4 *>(cols + 32 * mb + 16 * t + 8 * h);
          int4 b = *reinterpret_cast<const int4 *>(cols + 32 * mb + 16 * t + 8 * h + 4);
          keys[8 * t + 0] = a.x; keys[8 * t + 1] = a.y; keys[8 * t + 2] = a.z; keys[8 * t + 3] = a.w;
          keys[8 * t + 4] = b.x; keys[8 * t + 5] = b.y; keys[8 * t + 6] = b.z; keys[8 * t + 7] = b.w;
        }
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) keys[r] = kbase + 32 * mb + 16 * (r >> 3) + 8 * h + (r & 7);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = keys[r];
        bool okk = true;
        if (MODE == 1) okk = key >= mp.lo && key < mp.hi;
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
          const int qi = mp.q0 + 32 * nb + n;
          bool ok = okk && key <= qi;
          if (MODE == 1) ok = ok && (key < mp.n_init || key + mp.n_local > qi);
          s[mb][nb][r] = ok ? s[mb][nb][r] : -INFINITY;
        }
      }
    }
  }

  bf16x8 p[2][2][2];  // [nb][mb][t]
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    float mx = s[0][nb][0];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[mb][nb][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_old = st.m[nb];
    const float m_new = fmaxf(m_old, mx * c_log2);
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = fast_exp2(m_old - m_use);
    st.m[nb] = m_new;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
      st.l[nb] *= alpha;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.o[db][nb][r] *= alpha;
    }
    float lsum = 0.f;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        float e[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          e[i] = fast_exp2(fmaf(s[mb][nb][8 * t + i], c_log2, -m_use));
          lsum += e[i];
        }
        bf16x8 pk;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          f32x2 two = {e[2 * i], e[2 * i + 1]};
          bf16x2 b2 = __builtin_convertvector(two, bf16x2);
          pk[2 * i] = b2[0];
          pk[2 * i + 1] = b2[1];
        }
        p[nb][mb][t] = pk;
      }
    st.l[nb] += lsum;
  }

#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        bf16x8 a = *reinterpret_cast<const bf16x8 *>(ldsVt + (32 * db + n) * VT_PITCH + 32 * mb + 16 * t + 8 * h);
        st.o[db][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, p[0][mb][t], st.o[db][0], 0, 0, 0);
        st.o[db][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, p[1][mb][t], st.o[db][1], 0, 0, 0);
      }
}

// Classify a contiguous tile [kbase, kbase+64) for the wave whose rows are
// q0 .. q0+63.  Returns 0 = nothing to attend (skip), 1 = fully attended
// (no element mask needed), 2 = partially attended.
__device__ inline int classify_tile(int kbase, const MaskP &mp) {
  const int klast = kbase + BK - 1, qlast = mp.q0 + BQ - 1;
  if (klast < mp.lo || kbase >= mp.hi || kbase > qlast) return 0;
  if (kbase >= mp.n_init && klast + mp.n_local <= mp.q0) return 0;
  const bool full = kbase >= mp.lo && klast < mp.hi && klast <= mp.q0 &&
                    (klast < mp.n_init || kbase + mp.n_local > qlast);
  return full ? 1 : 2;
}

__device__ inline void contiguous_tile(WaveState &st, const bf16_t *ldsK, const bf16_t *ldsVt, int kbase,
                                       const MaskP &mp, float c_log2, int lane) {
  const int cls = classify_tile(kbase, mp);
  if (cls == 1)
    tile_compute<0>(st, ldsK, ldsVt, kbase, nullptr, mp, c_log2, lane);
  else if (cls == 2)
    tile_compute<1>(st, ldsK, ldsVt, kbase, nullptr, mp, c_log2, lane);
}

// Work-item decode shared by the kernels: heads are taken in chunks of 4
// list slots, and inside a chunk the block index varies slowest (descending,
// heaviest first), so that the workgroups resident on one XCD at a time are a
// few neighbouring query blocks of up to 4 heads (one GQA group when the head
// list is sorted) and share their K/V tiles in that XCD's L2.
__device__ inline void decode_item(int logical, int n_heads, int n_blk, int &slot, int &blk) {
  const int n_full = n_heads >> 2, rem = n_heads & 3;
  const int full_items = n_full * 4 * n_blk;
  int r;
  if (logical < full_items) {
    const int chunk = logical / (4 * n_blk);
    r = logical - chunk * 4 * n_blk;
    slot = chunk * 4 + (r & 3);
    r >>= 2;
  } else {
    r = logical - full_items;
    slot = n_full * 4 + r % rem;
    r = r / rem;
  }
  blk = n_blk - 1 - r;
}

// ---------------------------------------------------------------------------
// A-shape (and dense causal: n_init = 0, n_local >= N).  4 waves, 256 query
// rows of one head per workgroup; shared, double-buffered K/V tiles.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void ashape_kernel(QKV x, HeadList hl, int n_init, int n_local,
                                                     Sched sched) {
  extern __shared__ __attribute__((aligned(16))) bf16_t lds[];
  const int logical = logical_wg(sched);
  if (logical < 0) return;
  const int NB = x.N / BQ, NSB = (NB + 3) / 4;
  int slot, sb;
  decode_item(logical, hl.n, NSB, slot, sb);
  const int head = hl.h[slot], kvh = head / x.group;
  const bf16_t *qh = x.q + head * x.q_sh, *kh = x.k + kvh * x.k_sh, *vh = x.v + kvh * x.v_sh;
  bf16_t *oh = x.o + head * x.o_sh;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int blk = sb * 4 + wave;
  const bool active = blk < NB;
  const int q0 = (active ? blk : NB - 1) * BQ;   // inactive waves shadow the last block, write nothing

  WaveState st;
  wave_init(st, qh, x.q_st, q0, lane);
  MaskP mp;
  mp.q0 = q0; mp.lo = 0; mp.hi = x.N; mp.n_init = n_init; mp.n_local = n_local;

  // key ranges of the workgroup, 64-aligned: sink [0, e1) and window [s2, e2)
  const int wq0 = sb * 4 * BQ, wq1 = min(wq0 + 4 * BQ, x.N);
  int e1 = min(((n_init + BK - 1) / BK) * BK, wq1);
  int s2 = max(wq0 - n_local + 1, 0) / BK * BK;
  if (s2 <= e1) { s2 = 0; e1 = 0; }
  const int T1 = e1 / BK, T = T1 + (wq1 - s2) / BK;

  TileRegs<256> regs;
  auto tile_base = [&](int t) { return t < T1 ? t * BK : s2 + (t - T1) * BK; };
  tile_issue<256, true>(regs, kh, vh, x.k_st, x.v_st, tile_base(0), nullptr, x.N, tid);
  tile_store<256>(regs, lds, lds + K_TILE, tid);
  __syncthreads();
  for (int t = 0; t < T; ++t) {
    bf16_t *cur = lds + (t & 1) * STAGE, *nxt = lds + ((t + 1) & 1) * STAGE;
    if (t + 1 < T) tile_issue<256, true>(regs, kh, vh, x.k_st, x.v_st, tile_base(t + 1), nullptr, x.N, tid);
    contiguous_tile(st, cur, cur + K_TILE, tile_base(t), mp, x.c_log2, lane);
    if (t + 1 < T) tile_store<256>(regs, nxt, nxt + K_TILE, tid);
    __syncthreads();
  }
  // epilogue: each wave transposes its O tile through its own slice of LDS
  bf16_t *mine = lds + wave * K_TILE;
  if (active) wave_finish(st, oh, x.o_st, q0, mine, lane);
}

// ---------------------------------------------------------------------------
// Block-Sparse: one wave per (head, query block); tiles = listed key blocks.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void bs_kernel(QKV x, HeadList hl, const int32_t *blk_idx,
                                                const int32_t *blk_cnt, int topk, Sched sched) {
  extern __shared__ __attribute__((aligned(16))) bf16_t lds[];
  const int logical = logical_wg(sched);
  if (logical < 0) return;
  const int NB = x.N / BQ;
  int slot, b;
  decode_item(logical, hl.n, NB, slot, b);
  const int head = hl.h[slot], kvh = head / x.group;
  const bf16_t *qh = x.q + head * x.q_sh, *kh = x.k + kvh * x.k_sh, *vh = x.v + kvh * x.v_sh;
  bf16_t *oh = x.o + head * x.o_sh;
  const int lane = threadIdx.x;
  const int q0 = b * BQ;

  WaveState st;
  wave_init(st, qh, x.q_st, q0, lane);
  MaskP mp;
  mp.q0 = q0; mp.lo = 0; mp.hi = x.N; mp.n_init = KEY_NONE; mp.n_local = 1;

  const int32_t *list = blk_idx + ((int64_t)slot * NB + b) * topk;
  const int cnt = min(max(blk_cnt[(int64_t)slot * NB + b], 0), topk);
  bf16_t *ldsK = lds, *ldsVt = lds + K_TILE;

  TileRegs<64> regs;
  // next valid entry at or after position i (block ids outside [0, NB) are ignored)
  auto next_valid = [&](int i) {
    while (i < cnt) {
      int c = list[i];
      if (c >= 0 && c < NB) break;
      ++i;
    }
    return i;
  };
  int i = next_valid(0);
  if (i < cnt) tile_issue<64, true>(regs, kh, vh, x.k_st, x.v_st, list[i] * BK, nullptr, x.N, lane);
  while (i < cnt) {
    const int kbase = list[i] * BK;
    tile_store<64>(regs, ldsK, ldsVt, lane);
    __syncthreads();
    const int j = next_valid(i + 1);
    if (j < cnt) tile_issue<64, true>(regs, kh, vh, x.k_st, x.v_st, list[j] * BK, nullptr, x.N, lane);
    contiguous_tile(st, ldsK, ldsVt, kbase, mp, x.c_log2, lane);
    __syncthreads();
    i = j;
  }
  wave_finish(st, oh, x.o_st, q0, lds, lane);
}

// ---------------------------------------------------------------------------
// Vertical-Slash: one wave per (head, query block).
//  phase A: the slash runs [t0, t1) of the head, mapped to keys q0 - t, tiled
//           64 keys at a time from the run's first key;
//  phase B: kept verticals that are causal for the block and outside every
//           run, compacted (ballot + prefix count) into LDS and gathered 64 at
//           a time.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void vs_kernel(QKV x, HeadList hl, const int32_t *v_idx,
                                                const int32_t *cover, const uint32_t *cover_bits,
                                                const int32_t *counts, int nv, int ns, int cover_words,
                                                Sched sched) {
  extern __shared__ __attribute__((aligned(16))) bf16_t lds[];
  const int logical = logical_wg(sched);
  if (logical < 0) return;
  const int NB = x.N / BQ;
  int slot, b;
  decode_item(logical, hl.n, NB, slot, b);
  const int head = hl.h[slot], kvh = head / x.group;
  const bf16_t *qh = x.q + head * x.q_sh, *kh = x.k + kvh * x.k_sh, *vh = x.v + kvh * x.v_sh;
  bf16_t *oh = x.o + head * x.o_sh;
  const int lane = threadIdx.x;
  const int q0 = b * BQ;

  bf16_t *ldsK = lds, *ldsVt = lds + K_TILE;
  int *cols = reinterpret_cast<int *>(lds + STAGE);   // [VCAP + 64]

  const int n_v = min(max(counts[slot * 4 + 0], 0), nv);
  const int n_c = min(max(counts[slot * 4 + 2], 0), ns);
  const int32_t *vlist = v_idx + (int64_t)slot * nv;
  const int2 *runs = reinterpret_cast<const int2 *>(cover) + (int64_t)slot * ns;
  const uint32_t *bits = cover_bits + (int64_t)slot * cover_words;

  WaveState st;
  wave_init(st, qh, x.q_st, q0, lane);
  MaskP mp;
  mp.q0 = q0; mp.n_init = KEY_NONE; mp.n_local = 1; mp.lo = 0; mp.hi = 0;

  TileRegs<64> regs;

  // ---- phase A: slash runs -------------------------------------------------
  // state of the tile generator
  int iv = 0, ks = 0, ke = 0, pos = 0;   // run index, clipped key range [ks, ke), next tile start
  auto next_run_tile = [&](int &kbase, int &lo, int &hi) -> bool {
    while (true) {
      if (pos < ke) {
        kbase = pos; lo = ks; hi = ke;
        pos += BK;
        return true;
      }
      if (iv >= n_c) return false;
      const int2 r = runs[iv];
      if (r.x > q0) { iv = n_c; return false; }   // runs ascend: no later run reaches key >= 0
      ++iv;
      ks = max(q0 - r.y + 1, 0);
      ke = min(q0 - r.x + 1, x.N);
      pos = ks;
    }
  };
  int kb, lo, hi, kb2, lo2, hi2;
  bool have = next_run_tile(kb, lo, hi);
  if (have) tile_issue<64, true>(regs, kh, vh, x.k_st, x.v_st, kb, nullptr, x.N, lane);
  while (have) {
    tile_store<64>(regs, ldsK, ldsVt, lane);
    __syncthreads();
    const bool have2 = next_run_tile(kb2, lo2, hi2);
    if (have2) tile_issue<64, true>(regs, kh, vh, x.k_st, x.v_st, kb2, nullptr, x.N, lane);
    mp.lo = lo; mp.hi = hi;
    contiguous_tile(st, ldsK, ldsVt, kb, mp, x.c_log2, lane);
    __syncthreads();
    have = have2; kb = kb2; lo = lo2; hi = hi2;
  }

  // ---- phase B: verticals ----------------------------------------------------
  const int qlast = q0 + BQ - 1;
  int vpos = 0;                       // next entry of vlist to examine
  while (vpos < n_v) {
    // compact up to VCAP columns into cols[]
    int ncol = 0;
    while (vpos < n_v && ncol <= VCAP - 64) {
      const int i = vpos + lane;
      int v = i < n_v ? vlist[i] : KEY_NONE;
      bool ok = v <= qlast && v >= 0;
      if (ok) {
        const int t = q0 - v + 64;     // bit index of offset t = q0 - v, in [1, q0 + 64]
        ok = ((bits[t >> 5] >> (t & 31)) & 1u) == 0u;
      }
      const unsigned long long bal = __builtin_amdgcn_ballot_w64(ok);
      const int before = __builtin_popcountll(bal & ((1ull << lane) - 1ull));
      if (ok) cols[ncol + before] = v;
      ncol += __builtin_popcountll(bal);
      vpos += 64;
      // the list ascends: once a whole chunk is past the block nothing follows
      const int vfirst = __shfl(v, 0);
      if (vfirst > qlast) { vpos = n_v; break; }
    }
    if (ncol == 0) continue;
    const int ntile = (ncol + BK - 1) / BK;
    if (lane + ncol < ntile * BK) cols[ncol + lane] = KEY_NONE;   // pad the last tile
    __syncthreads();
    tile_issue<64, false>(regs, kh, vh, x.k_st, x.v_st, 0, cols, x.N, lane);
    for (int t = 0; t < ntile; ++t) {
      tile_store<64>(regs, ldsK, ldsVt, lane);
      __syncthreads();
      if (t + 1 < ntile)
        tile_issue<64, false>(regs, kh, vh, x.k_st, x.v_st, 0, cols + (t + 1) * BK, x.N, lane);
      tile_compute<2>(st, ldsK, ldsVt, 0, cols + t * BK, mp, x.c_log2, lane);
      __syncthreads();
    }
  }
  wave_finish(st, oh, x.o_st, q0, lds, lane);
}

// ---------------------------------------------------------------------------
// host-side launches
// ---------------------------------------------------------------------------
static hipError_t set_lds(const void *fn, size_t bytes) {
  return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

hipError_t launch_ashape(const QKV &x, const HeadList &hl, int n_init, int n_local, hipStream_t st) {
  const int NB = x.N / BQ, NSB = (NB + 3) / 4;
  const Sched s = make_sched((int64_t)hl.n * NSB);
  const size_t lds = 2 * STAGE * sizeof(bf16_t);
  hipError_t e = set_lds(reinterpret_cast<const void *>(ashape_kernel), lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(ashape_kernel, dim3(s.per_xcd * 8), dim3(256), lds, st, x, hl, n_init, n_local, s);
  return hipGetLastError();
}

hipError_t launch_bs(const QKV &x, const HeadList &hl, const int32_t *blk_idx, const int32_t *blk_cnt,
                     int topk, hipStream_t st) {
  const int NB = x.N / BQ;
  const Sched s = make_sched((int64_t)hl.n * NB);
  const size_t lds = STAGE * sizeof(bf16_t);
  hipError_t e = set_lds(reinterpret_cast<const void *>(bs_kernel), lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(bs_kernel, dim3(s.per_xcd * 8), dim3(64), lds, st, x, hl, blk_idx, blk_cnt, topk, s);
  return hipGetLastError();
}

hipError_t launch_vs(const QKV &x, const HeadList &hl, const int32_t *v_idx, const int32_t *cover,
                     const uint32_t *cover_bits, const int32_t *counts, int nv, int ns,
                     int cover_words, hipStream_t st) {
  const int NB = x.N / BQ;
  const Sched s = make_sched((int64_t)hl.n * NB);
  const size_t lds = STAGE * sizeof(bf16_t) + (VCAP + 64) * sizeof(int);
  hipError_t e = set_lds(reinterpret_cast<const void *>(vs_kernel), lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(vs_kernel, dim3(s.per_xcd * 8), dim3(64), lds, st, x, hl, v_idx, cover, cover_bits,
                     counts, nv, ns, cover_words, s);
  return hipGetLastError();
}

}  // namespace minf
