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
//  * Per key tile the wave computes S^T = K Q^T with v_mfma_f32_32x32x16_bf16
//    (keys on the M axis).  The accumulator layout of S^T is exactly the
//    B-operand layout the second contraction O^T += V^T P^T needs, so P never
//    leaves registers: no LDS round trip, no cross-lane shuffles for P.  The
//    only cross-lane traffic of the softmax is one exchange between lanes l and
//    l^32 per 32 query rows for the row max.
//  * K and V tiles go global -> LDS directly (global_load_lds_dwordx4), row
//    major with an XOR chunk swizzle; the K operand is a 16-byte LDS read, the
//    V^T operand comes from the transposing LDS read ds_read_b64_tr_b16.  No
//    VGPR staging, no LDS store instructions, no register transposes.
//  * Tiles are fetched by key index, so a gathered tile of vertical columns
//    costs the same as a contiguous one.  No mask tensor exists anywhere: the
//    element mask is evaluated from (query row, key id) in registers, and only
//    on tiles that can contain a masked element.
//  * The running max is refreshed lazily: O and l are rescaled only when some
//    row's max grew by more than 2^8 since the last refresh; exponentials are
//    taken against the stale max (at most 2^8, harmless in fp32 / bf16).
//  * A-shape / dense: a workgroup is 4 waves = 4 consecutive query blocks of
//    one head; 64-key K/V tiles are staged once in LDS (double buffered) and
//    shared by the 4 waves.  Block-Sparse / Vertical-Slash: tile lists differ
//    per query block, so a workgroup is a single wave that streams 32-key
//    steps through a private double buffer; 4 workgroups share a CU.
#include "mfma_tile.h"

namespace minf {

constexpr int VCAP = 1024;               // compacted vertical columns held in LDS per round
constexpr int TILE_BYTES = 64 * ROW_BYTES;   // 64 rows of K or of V
constexpr int HALF_BYTES = 32 * ROW_BYTES;   // 32 rows
constexpr float RESCALE_LOG2 = 8.0f;     // refresh the running max when it grows by more than 2^8

struct WaveState {
  bf16x8 q[2][8];     // Q fragments: [query half nb][k step]: Q[32nb + n][16ks + 8h ..]
  f32x16 o[4][2];     // O^T accumulators: [d block][query half]
  float m[2];         // reference max of the scaled logits (log2 domain) of query 32nb + n
  float l[2];         // this lane's share of the running row sum
};

// Element mask of a step, as seen by one wave (all fields wave-uniform).
// A key is attended by query row i iff lo <= key < hi, key <= i and
// (key < n_init or key + n_local > i).
struct MaskP {
  int q0;             // first query row of the wave's block
  int lo, hi;
  int n_init, n_local;
};

#define MINF_WAIT_VMCNT(n) asm volatile("s_waitcnt vmcnt(" #n ")" ::: "memory")

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

// Normalise, convert to bf16, transpose through 16 KiB of LDS owned by this
// wave and write O rows with 16-byte coalesced stores.
__device__ inline void wave_finish(WaveState &st, bf16_t *oh, int64_t o_st, int q0, char *lds, int lane) {
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
        w.x = __builtin_bit_cast(unsigned, pa);
        w.y = __builtin_bit_cast(unsigned, pb);
        *reinterpret_cast<uint2 *>(lds + swz_byte(32 * nb + n, 4 * db + g) + 8 * h) = w;
      }
  }
  // LDS operations of one wave execute in issue order; the fences only keep the
  // compiler from moving the reads below above the writes of other lanes.
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int c = lane + 64 * i;
    const int row = c >> 4, col = c & 15;
    const uint4 w = *reinterpret_cast<const uint4 *>(lds + swz_byte(row, col));
    *reinterpret_cast<uint4 *>(oh + (int64_t)(q0 + row) * o_st + col * 8) = w;
  }
}

// ---- one step of MB * 32 keys: S^T = K Q^T, mask, online softmax, O^T += V^T P^T
// MODE 0: no element is masked.  MODE 1: contiguous keys kbase + idx, mask mp.
// MODE 2: gathered keys cols[idx] (LDS), attended iff key <= query row.
// Register r of s[mb][nb] holds key index 32mb + 16(r/8) + 8h + (r%8) and
// query 32nb + n (n = lane%32, h = lane/32).
template <int MB, int MODE>
__device__ inline void step_compute(WaveState &st, const LaneOfs &lo, const char *tK, const char *tV,
                                    int kbase, const int *cols, const MaskP &mp, float c_log2, int lane) {
  const int n = lane & 31, h = lane >> 5;
  f32x16 s[MB][2];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[mb][nb][r] = 0.f;

#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const bf16x8 a = lds_read_k(tK, lo.k[ks] + mb * HALF_BYTES);
      s[mb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, st.q[0][ks], s[mb][0], 0, 0, 0);
      s[mb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, st.q[1][ks], s[mb][1], 0, 0, 0);
    }
  }

  if (MODE != 0) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      int keys[16];
      if (MODE == 2) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const int4 a = *reinterpret_cast<const int4 *>(cols + 32 * mb + 16 * t + 8 * h);
          const int4 b = *reinterpret_cast<const int4 *>(cols + 32 * mb + 16 * t + 8 * h + 4);
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

  bf16x8 p[2][MB][2];  // [nb][mb][t]
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    float mx = s[0][nb][0];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[mb][nb][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32)) * c_log2;
    // lazy refresh of the reference max (wave-uniform decision)
    if (__builtin_amdgcn_ballot_w64(mx > st.m[nb] + RESCALE_LOG2) != 0) {
      const float m_old = st.m[nb];
      const float m_new = fmaxf(m_old, mx);
      const float alpha = fast_exp2(m_old - (m_new == -INFINITY ? 0.f : m_new));
      st.m[nb] = m_new;
      st.l[nb] *= alpha;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.o[db][nb][r] *= alpha;
    }
    const float m_use = st.m[nb] == -INFINITY ? 0.f : st.m[nb];
    float lsum = 0.f;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
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
          const f32x2 two = {e[2 * i], e[2 * i + 1]};
          const bf16x2 b2 = __builtin_convertvector(two, bf16x2);
          pk[2 * i] = b2[0];
          pk[2 * i + 1] = b2[1];
        }
        p[nb][mb][t] = pk;
      }
    st.l[nb] += lsum;
  }

#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const int base = (32 * mb + 16 * t) * ROW_BYTES;
        const bf16x8 a = lds_read_vt(tV, lo.v[db][0] + base, lo.v[db][1] + base);
        st.o[db][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, p[0][mb][t], st.o[db][0], 0, 0, 0);
        st.o[db][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, p[1][mb][t], st.o[db][1], 0, 0, 0);
      }
}

// Classify a contiguous step [kbase, kbase + W) for the wave whose rows are
// q0 .. q0+63.  0 = nothing to attend (skip), 1 = fully attended (no element
// mask needed), 2 = partially attended.
template <int W>
__device__ inline int classify_step(int kbase, const MaskP &mp) {
  const int klast = kbase + W - 1, qlast = mp.q0 + BQ - 1;
  if (klast < mp.lo || kbase >= mp.hi || kbase > qlast) return 0;
  if (kbase >= mp.n_init && klast + mp.n_local <= mp.q0) return 0;
  const bool full = kbase >= mp.lo && klast < mp.hi && klast <= mp.q0 &&
                    (klast < mp.n_init || kbase + mp.n_local > qlast);
  return full ? 1 : 2;
}

template <int MB>
__device__ inline void contiguous_step(WaveState &st, const LaneOfs &lo, const char *tK, const char *tV,
                                       int kbase, const MaskP &mp, float c_log2, int lane) {
  const int cls = classify_step<32 * MB>(kbase, mp);
  if (cls == 1)
    step_compute<MB, 0>(st, lo, tK, tV, kbase, nullptr, mp, c_log2, lane);
  else if (cls == 2)
    step_compute<MB, 1>(st, lo, tK, tV, kbase, nullptr, mp, c_log2, lane);
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
// rows of one head per workgroup; shared, double-buffered 64-key K/V tiles.
// LDS: 2 stages x (K 16 KiB + V 16 KiB).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void ashape_kernel(QKV x, HeadList hl, int n_init, int n_local,
                                                     Sched sched) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int logical = logical_wg(sched);
  if (logical < 0) return;
  const int NB = x.N / BQ, NSB = (NB + 3) / 4;
  int slot, sb;
  decode_item(logical, hl.n, NSB, slot, sb);
  const int head = hl.h[slot], kvh = head / x.group;
  const bf16_t *qh = x.q + head * x.q_sh, *kh = x.k + kvh * x.k_sh, *vh = x.v + kvh * x.v_sh;
  bf16_t *oh = x.o + head * x.o_sh;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int blk = sb * 4 + wave;
  const bool active = blk < NB;
  const int q0 = (active ? blk : NB - 1) * BQ;   // an idle wave shadows the last block, writes nothing

  WaveState st;
  wave_init(st, qh, x.q_st, q0, lane);
  LaneOfs lo;
  lane_offsets(lo, lane);
  MaskP mp;
  mp.q0 = q0; mp.lo = 0; mp.hi = x.N; mp.n_init = n_init; mp.n_local = n_local;

  // key ranges of the workgroup, 64-aligned: sink [0, e1) and window [s2, e2)
  const int wq0 = sb * 4 * BQ, wq1 = min(wq0 + 4 * BQ, x.N);
  int e1 = min(((n_init + BK - 1) / BK) * BK, wq1);
  int s2 = max(wq0 - n_local + 1, 0) / BK * BK;
  if (s2 <= e1) { s2 = 0; e1 = 0; }
  const int T1 = e1 / BK, T = T1 + (wq1 - s2) / BK;
  auto tile_base = [&](int t) { return t < T1 ? t * BK : s2 + (t - T1) * BK; };
  auto fetch = [&](int t) {
    char *stg = lds + (t & 1) * 2 * TILE_BYTES;
    dma_rows<4, 64, true>(kh, x.k_st, tile_base(t), nullptr, x.N, stg, wave, lane);
    dma_rows<4, 64, true>(vh, x.v_st, tile_base(t), nullptr, x.N, stg + TILE_BYTES, wave, lane);
  };

  fetch(0);
  MINF_WAIT_VMCNT(0);
  __syncthreads();
  for (int t = 0; t < T; ++t) {
    if (t + 1 < T) fetch(t + 1);
    const char *stg = lds + (t & 1) * 2 * TILE_BYTES;
    contiguous_step<2>(st, lo, stg, stg + TILE_BYTES, tile_base(t), mp, x.c_log2, lane);
    MINF_WAIT_VMCNT(0);
    __syncthreads();
  }
  if (active) wave_finish(st, oh, x.o_st, q0, lds + wave * TILE_BYTES, lane);
}

// ---------------------------------------------------------------------------
// Single-wave kernels: 32-key steps through a private double buffer.
// LDS: 2 stages x (K 8 KiB + V 8 KiB) = 32 KiB (+ column list for VS).
// One step = 16 global_load_lds instructions (8 K + 8 V); the wave keeps the
// next step's loads in flight while it computes the current one.
// ---------------------------------------------------------------------------
struct StepBuf {
  char *lds;
  __device__ inline char *k(int s) const { return lds + s * 2 * HALF_BYTES; }
  __device__ inline char *v(int s) const { return lds + s * 2 * HALF_BYTES + HALF_BYTES; }
};

template <bool CONTIG>
__device__ inline void fetch_step(const StepBuf &sb, int s, const bf16_t *kh, const bf16_t *vh, int64_t k_st,
                                  int64_t v_st, int kbase, const int *cols, int N, int lane) {
  dma_rows<1, 32, CONTIG>(kh, k_st, kbase, cols, N, sb.k(s), 0, lane);
  dma_rows<1, 32, CONTIG>(vh, v_st, kbase, cols, N, sb.v(s), 0, lane);
}

// ---------------------------------------------------------------------------
// Block-Sparse: one wave per (head, query block); steps = halves of the listed
// key blocks.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void bs_kernel(QKV x, HeadList hl, const int32_t *blk_idx,
                                                const int32_t *blk_cnt, int topk, Sched sched) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
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
  LaneOfs lo;
  lane_offsets(lo, lane);
  MaskP mp;
  mp.q0 = q0; mp.lo = 0; mp.hi = x.N; mp.n_init = KEY_NONE; mp.n_local = 1;
  const StepBuf buf{lds};

  const int32_t *list = blk_idx + ((int64_t)slot * NB + b) * topk;
  const int cnt = min(max(blk_cnt[(int64_t)slot * NB + b], 0), topk);
  // step index u = 2 * (list position) + half; entries outside [0, NB) are skipped
  auto next_valid = [&](int i) {
    while (i < cnt) {
      const int c = list[i];
      if (c >= 0 && c < NB) break;
      ++i;
    }
    return i;
  };
  int i = next_valid(0), half = 0, s = 0;
  if (i < cnt) fetch_step<true>(buf, 0, kh, vh, x.k_st, x.v_st, list[i] * BK, nullptr, x.N, lane);
  while (i < cnt) {
    const int kbase = list[i] * BK + 32 * half;
    int i2 = i, half2 = half ^ 1;
    if (half == 1) i2 = next_valid(i + 1);
    if (i2 < cnt) {
      fetch_step<true>(buf, s ^ 1, kh, vh, x.k_st, x.v_st, list[i2] * BK + 32 * half2, nullptr, x.N, lane);
      MINF_WAIT_VMCNT(16);
    } else {
      MINF_WAIT_VMCNT(0);
    }
    contiguous_step<1>(st, lo, buf.k(s), buf.v(s), kbase, mp, x.c_log2, lane);
    i = i2; half = half2; s ^= 1;
  }
  wave_finish(st, oh, x.o_st, q0, lds, lane);
}

// ---------------------------------------------------------------------------
// Vertical-Slash: one wave per (head, query block).
//  phase A: the slash runs [t0, t1) of the head, mapped to keys q0 - t, walked
//           32 keys at a time from the run's first key;
//  phase B: kept verticals that are causal for the block and outside every
//           run, compacted (ballot + prefix count) into LDS and gathered 32 at
//           a time.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void vs_kernel(QKV x, HeadList hl, const int32_t *v_idx,
                                                const int32_t *cover, const uint32_t *cover_bits,
                                                const int32_t *counts, int nv, int ns, int cover_words,
                                                Sched sched) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
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

  const StepBuf buf{lds};
  int *cols = reinterpret_cast<int *>(lds + 4 * HALF_BYTES);   // [VCAP + 64]

  const int n_v = min(max(counts[slot * 4 + 0], 0), nv);
  const int n_c = min(max(counts[slot * 4 + 2], 0), ns);
  const int32_t *vlist = v_idx + (int64_t)slot * nv;
  const int2 *runs = reinterpret_cast<const int2 *>(cover) + (int64_t)slot * ns;
  const uint32_t *bits = cover_bits + (int64_t)slot * cover_words;

  WaveState st;
  wave_init(st, qh, x.q_st, q0, lane);
  LaneOfs lo;
  lane_offsets(lo, lane);
  MaskP mp;
  mp.q0 = q0; mp.n_init = KEY_NONE; mp.n_local = 1; mp.lo = 0; mp.hi = 0;

  // ---- phase A: slash runs -------------------------------------------------
  int iv = 0, ks = 0, ke = 0, pos = 0;   // run index, clipped key range [ks, ke), next step start
  auto next_run_step = [&](int &kbase, int &rlo, int &rhi) -> bool {
    while (true) {
      if (pos < ke) {
        kbase = pos; rlo = ks; rhi = ke;
        pos += 32;
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
  int s = 0;
  int kb, rlo, rhi, kb2, rlo2, rhi2;
  bool have = next_run_step(kb, rlo, rhi);
  if (have) fetch_step<true>(buf, 0, kh, vh, x.k_st, x.v_st, kb, nullptr, x.N, lane);
  while (have) {
    const bool have2 = next_run_step(kb2, rlo2, rhi2);
    if (have2) {
      fetch_step<true>(buf, s ^ 1, kh, vh, x.k_st, x.v_st, kb2, nullptr, x.N, lane);
      MINF_WAIT_VMCNT(16);
    } else {
      MINF_WAIT_VMCNT(0);
    }
    mp.lo = rlo; mp.hi = rhi;
    contiguous_step<1>(st, lo, buf.k(s), buf.v(s), kb, mp, x.c_log2, lane);
    have = have2; kb = kb2; rlo = rlo2; rhi = rhi2; s ^= 1;
  }

  // ---- phase B: verticals ----------------------------------------------------
  const int qlast = q0 + BQ - 1;
  int vpos = 0;                       // next entry of vlist to examine
  while (vpos < n_v) {
    // compact up to VCAP columns into cols[]
    int ncol = 0;
    while (vpos < n_v && ncol <= VCAP - 64) {
      const int i = vpos + lane;
      const int v = i < n_v ? vlist[i] : KEY_NONE;
      bool ok = v <= qlast && v >= 0;
      if (ok) {
        const int t = q0 - v + 64;     // bit index of offset q0 - v, in [1, q0 + 64]
        ok = ((bits[t >> 5] >> (t & 31)) & 1u) == 0u;
      }
      const unsigned long long bal = __builtin_amdgcn_ballot_w64(ok);
      const int before = __builtin_popcountll(bal & ((1ull << lane) - 1ull));
      if (ok) cols[ncol + before] = v;
      ncol += __builtin_popcountll(bal);
      vpos += 64;
      // the list ascends: once a whole chunk is past the block nothing follows
      if (__shfl(v, 0) > qlast) { vpos = n_v; break; }
    }
    if (ncol == 0) continue;
    const int nstep = (ncol + 31) / 32;
    if (lane + ncol < nstep * 32) cols[ncol + lane] = KEY_NONE;   // pad the last step
    __syncthreads();                   // cols[] visible to every lane; earlier vector loads drained
    fetch_step<false>(buf, s, kh, vh, x.k_st, x.v_st, 0, cols, x.N, lane);
    for (int t = 0; t < nstep; ++t) {
      if (t + 1 < nstep) {
        fetch_step<false>(buf, s ^ 1, kh, vh, x.k_st, x.v_st, 0, cols + (t + 1) * 32, x.N, lane);
        MINF_WAIT_VMCNT(16);
      } else {
        MINF_WAIT_VMCNT(0);
      }
      step_compute<1, 2>(st, lo, buf.k(s), buf.v(s), 0, cols + t * 32, mp, x.c_log2, lane);
      s ^= 1;
    }
    __syncthreads();                   // every lane is done with cols[] before the next round refills it
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
  const size_t lds = 4 * TILE_BYTES;
  hipError_t e = set_lds(reinterpret_cast<const void *>(ashape_kernel), lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(ashape_kernel, dim3(s.per_xcd * 8), dim3(256), lds, st, x, hl, n_init, n_local, s);
  return hipGetLastError();
}

hipError_t launch_bs(const QKV &x, const HeadList &hl, const int32_t *blk_idx, const int32_t *blk_cnt,
                     int topk, hipStream_t st) {
  const int NB = x.N / BQ;
  const Sched s = make_sched((int64_t)hl.n * NB);
  const size_t lds = 4 * HALF_BYTES;
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
  const size_t lds = 4 * HALF_BYTES + (VCAP + 64) * sizeof(int);
  hipError_t e = set_lds(reinterpret_cast<const void *>(vs_kernel), lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(vs_kernel, dim3(s.per_xcd * 8), dim3(64), lds, st, x, hl, v_idx, cover, cover_bits,
                     counts, nv, ns, cover_words, s);
  return hipGetLastError();
}

}  // namespace minf
