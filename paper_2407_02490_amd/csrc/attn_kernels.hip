// Causal sparse attention kernels for gfx950 (MI355X).
//
// What is computed: Eq. 1 of the paper, A(M) = softmax(QK^T/sqrt(d) - c(1-M)) V
// with c -> infinity, for the A-shape, Block-Sparse (App. C.4.1) and
// Vertical-Slash (App. C.4.2, Alg. 5) masks; the online-softmax recurrence of
// Alg. 5 (running max m, running sum l, rescale by exp(m - m_new)) is replaced
// by a fixed exponent reference with an exact fallback (below).
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
//  * Optimistic fixed reference: the exponent reference m of a row is taken
//    once, from the row max of the first step the wave computes, and is never
//    changed inside the hot loop: p = exp2(s - m) may then exceed 1, which fp32
//    accumulators and bf16 P (fp32 exponent range) absorb up to 2^100.  The
//    result is identical up to rounding because m cancels in O / l.  No
//    per-step row max, no rescale of the 128 O registers, no branch on data.
//    If a row sum ends up >= 2^100 or non-finite (logits that outgrow the first
//    step's max by more than ~69 nats) or below 2^-100 (every term underflowed:
//    logits far below the reference), the whole query block is redone with the
//    exact two-pass scheme: pass 1 finds every row max, pass 2 accumulates.
//  * Three tiles in flight per loop iteration: logits of tile t+1, softmax of
//    tile t, output update of tile t-1.  With one wave per SIMD (the kernels
//    need about 450 registers) the wave issues one instruction every four
//    cycles, in order, so the loops are built to an instruction budget: one
//    MFMA per issue group, logits accumulated in vector registers (reading
//    accumulator registers queues behind the MFMAs), Q and the LDS operands
//    in accumulator registers, scalar bookkeeping between MFMAs, constant
//    wait counts.
//  * A-shape / dense: a workgroup is 4 waves = 4 consecutive query blocks of
//    one head; 64-key K/V tiles go through LDS rings (four slots each, three
//    tiles live) shared by the 4 waves.  Block-Sparse / Vertical-Slash: tile
//    lists differ per query block, so a workgroup is a single wave that streams
//    32-key steps through private rings (2 K + 3 V slots, 40 KiB); 4 workgroups
//    share a CU.  Both loops are unrolled over their rings (4x and 6x), so that
//    every LDS slot address is an immediate.
#include <stdlib.h>
#include <string.h>
#include <type_traits>

#include "mfma_tile.h"
#include "vs_ring_sched.h"

namespace minf {

constexpr int VCAP = 1024;               // compacted vertical columns held in LDS per round
constexpr float L_LIMIT = 1.2676506e30f;  // 2^100: beyond it the optimistic pass is redone exactly
constexpr float L_TINY = 7.888609e-31f;   // 2^-100: below it too (underflow of every term of a row)

struct WaveState {
  bf16x8 q[2][8];     // Q fragments: [query half nb][k step]: Q[32nb + n][16ks + 8h ..]
  f32x16 o[4][2];     // O^T accumulators: [d block][query half]
  float m[2];         // exponent reference of query 32nb + n (scaled logits, log2 domain)
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


// ---- per-wave setup / epilogue ---------------------------------------------
__device__ inline void set_reference(WaveState &st, int nb, float m) { st.m[nb] = m; }

__device__ inline void load_q(WaveState &st, const bf16_t *qh, int64_t q_st, int q0, int lane) {
  const int n = lane & 31, h = lane >> 5;
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    const bf16_t *row = qh + (int64_t)(q0 + 32 * nb + n) * q_st + 8 * h;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) st.q[nb][ks] = *reinterpret_cast<const bf16x8 *>(row + 16 * ks);
  }
}

__device__ inline void wave_init(WaveState &st, const bf16_t *qh, int64_t q_st, int q0, int lane) {
  load_q(st, qh, q_st, q0, lane);
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    set_reference(st, nb, 0.f);
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

// ---- one step of MB * 32 keys: S^T = K Q^T, mask, p = exp2(c s - m), O^T += V^T P^T
// The MFMA sequences appear exactly once per loop that calls this function;
// everything that varies from step to step is a wave-uniform run-time flag that
// only touches the logits, so the O accumulators keep one home for the whole
// loop:
//   mask_mode 0: no element is masked; 1: keys kbase + idx with the mask mp
//   (GATHER: keys cols[idx] from LDS, attended iff key <= query row, always masked);
//   first: take the reference m from this step's row max (optimistic pass).
// PASS_MAX: only fold the row max into the reference candidates (st.l as scratch).
// Register r of s[mb][nb] holds key index 32mb + 16(r/8) + 8h + (r%8) and
// query 32nb + n (n = lane%32, h = lane/32).
enum { PASS_OPT = 0, PASS_MAX = 1, PASS_FIX = 2 };

template <int MB, bool GATHER, int PASS>
__device__ inline void step_compute(WaveState &st, const LaneOfs &lo, const char *tK, const char *tV,
                                    int kbase, const int *cols, const MaskP &mp, int mask_mode, bool first,
                                    float c_log2, int lane) {
  const int n = lane & 31, h = lane >> 5;
  f32x16 s[MB][2];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const bf16x8 a = lds_read_k(tK, lo.k[ks] + mb * HALF_BYTES);
      if (ks == 0) {
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        s[mb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, st.q[0][0], zero, 0, 0, 0);
        s[mb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, st.q[1][0], zero, 0, 0, 0);
      } else {
        s[mb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, st.q[0][ks], s[mb][0], 0, 0, 0);
        s[mb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, st.q[1][ks], s[mb][1], 0, 0, 0);
      }
    }
  }

  if (GATHER || mask_mode != 0) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      int keys[16];
      if (GATHER) {
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
        if (!GATHER) okk = key >= mp.lo && key < mp.hi;
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
          const int qi = mp.q0 + 32 * nb + n;
          bool ok = okk && key <= qi;
          if (!GATHER) ok = ok && (key < mp.n_init || key + mp.n_local > qi);
          s[mb][nb][r] = ok ? s[mb][nb][r] : -INFINITY;
        }
      }
    }
  }

  if (PASS == PASS_MAX) {
    // st.l collects the row max of the raw logits (scaled after the pass)
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      float mx = st.l[nb];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[mb][nb][r]);
      st.l[nb] = mx;
    }
    return;
  }

  if (PASS == PASS_OPT && first) {
    // take the reference from this step's row max
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      float mx = s[0][nb][0];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[mb][nb][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32)) * c_log2;
      set_reference(st, nb, mx == -INFINITY ? 0.f : mx);   // a row with no key yet: neutral reference
    }
  }

  bf16x8 p[2][MB][2];  // [nb][mb][t]
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    const float m_use = st.m[nb];
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

// ---- the same arithmetic as step_compute, split into its three phases so that a
// loop can overlap phases of neighbouring tiles (software pipelining) ---------
template <int MB>
__device__ inline void qk_tile(f32x16 (&s)[MB][2], const WaveState &st, const LaneOfs &lo, const char *tK) {
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const bf16x8 a = lds_read_k(tK, lo.k[ks] + mb * HALF_BYTES);
      if (ks == 0) {
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        s[mb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, st.q[0][0], zero, 0, 0, 0);
        s[mb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, st.q[1][0], zero, 0, 0, 0);
      } else {
        s[mb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, st.q[0][ks], s[mb][0], 0, 0, 0);
        s[mb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, st.q[1][ks], s[mb][1], 0, 0, 0);
      }
    }
  }
}

// Rare path on fresh logits of a contiguous tile: element mask and / or taking
// the exponent reference from this tile's row max.
template <int MB>
__device__ inline void special_tile(f32x16 (&s)[MB][2], WaveState &st, int kbase, const MaskP &mp,
                                    bool need_mask, bool first, float c_log2, int lane) {
  const int n = lane & 31, h = lane >> 5;
  if (need_mask) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = kbase + 32 * mb + 16 * (r >> 3) + 8 * h + (r & 7);
        const bool okk = key >= mp.lo && key < mp.hi;
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
          const int qi = mp.q0 + 32 * nb + n;
          const bool ok = okk && key <= qi && (key < mp.n_init || key + mp.n_local > qi);
          s[mb][nb][r] = ok ? s[mb][nb][r] : -INFINITY;
        }
      }
  }
  if (first) {
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      float mx = s[0][nb][0];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[mb][nb][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32)) * c_log2;
      set_reference(st, nb, mx == -INFINITY ? 0.f : mx);
    }
  }
}

// Cheap element mask for steps whose only constraints are a key window and
// causality (Block-Sparse, Vertical-Slash, dense): attended iff
// lo <= key < min(hi, query row + 1), one unsigned compare per element.
template <int MB>
__device__ inline void window_mask(f32x16 (&s)[MB][2], int kbase, const MaskP &mp, int lane) {
  const int n = lane & 31, h = lane >> 5;
  const int rel = kbase + 8 * h - mp.lo;                       // key - lo for index 0 of this lane
  unsigned span[2];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) span[nb] = (unsigned)max(min(mp.hi, mp.q0 + 32 * nb + n + 1) - mp.lo, 0);
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const unsigned d = (unsigned)(rel + 32 * mb + 16 * (r >> 3) + (r & 7));
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) s[mb][nb][r] = d < span[nb] ? s[mb][nb][r] : -INFINITY;
    }
}

template <int MB>
__device__ inline void softmax_tile(bf16x8 (&p)[2][MB][2], WaveState &st, const f32x16 (&s)[MB][2],
                                    float c_log2) {
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    const float m_use = st.m[nb];
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
}

// O^T += V^T P^T for one step.  The V^T operands are fetched from LDS two
// MFMA pairs ahead of their use (each pair runs 64 cycles, an LDS read takes
// longer than that to return).
template <int MB>
__device__ inline void pv_tile(WaveState &st, const LaneOfs &lo, const char *tV, const bf16x8 (&p)[2][MB][2]) {
  constexpr int NSTEP = MB * 2 * 4;      // (mb, t, db)
  constexpr int AHEAD = 2;
  bf16x8 a[NSTEP];
  auto fetch = [&](int i) {
    const int mb = i / 8, t = (i / 4) & 1, db = i & 3;
    const int base = (32 * mb + 16 * t) * ROW_BYTES;
    return lds_read_vt(tV, lo.v[db][0] + base, lo.v[db][1] + base);
  };
#pragma unroll
  for (int i = 0; i < AHEAD; ++i) a[i] = fetch(i);
#pragma unroll
  for (int i = 0; i < NSTEP; ++i) {
    if (i + AHEAD < NSTEP) a[i + AHEAD] = fetch(i + AHEAD);
    const int mb = i / 8, t = (i / 4) & 1, db = i & 3;
    st.o[db][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], p[0][mb][t], st.o[db][0], 0, 0, 0);
    st.o[db][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], p[1][mb][t], st.o[db][1], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// QK of one step fused with the softmax of the previous step, interleaved by
// hand: 8 rounds of {the 2 MB MFMAs of k-step ks; one eighth of the exp work;
// LDS reads of k-step ks+1}.  The vector ALU work of a round runs in the shadow
// of the round's MFMAs (32 cycles each).  sched_barrier(0) keeps the compiler
// from regrouping the rounds.
template <int MB>
__device__ inline void fused_qk_softmax(f32x16 (&s_nxt)[MB][2], bf16x8 (&p)[2][MB][2], WaveState &st,
                                        const f32x16 (&s_cur)[MB][2], const LaneOfs &lo, const char *tK,
                                        float c_log2) {
  constexpr int EPR = 4 * MB;            // logits per lane handled per round
  const float m0 = st.m[0], m1 = st.m[1];
  float lsum0 = 0.f, lsum1 = 0.f;
  bf16x8 a[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) a[mb] = lds_read_k(tK, lo.k[0] + mb * HALF_BYTES);
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    bf16x8 c[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      c[mb] = a[mb];
      if (ks + 1 < 8) a[mb] = lds_read_k(tK, lo.k[ks + 1] + mb * HALF_BYTES);
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      if (ks == 0) {
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        s_nxt[mb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(c[mb], st.q[0][0], zero, 0, 0, 0);
        s_nxt[mb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(c[mb], st.q[1][0], zero, 0, 0, 0);
      } else {
        s_nxt[mb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(c[mb], st.q[0][ks], s_nxt[mb][0], 0, 0, 0);
        s_nxt[mb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(c[mb], st.q[1][ks], s_nxt[mb][1], 0, 0, 0);
      }
    }
    // softmax slice ks of the previous step; logits are walked in the order [nb][mb][r]
#pragma unroll
    for (int i = 0; i < EPR; i += 2) {
      const int e = ks * EPR + i;
      const int nb = e / (16 * MB), mb = (e % (16 * MB)) / 16, r = e % 16;
      const float m_use = nb == 0 ? m0 : m1;
      const float e0 = fast_exp2(fmaf(s_cur[mb][nb][r], c_log2, -m_use));
      const float e1 = fast_exp2(fmaf(s_cur[mb][nb][r + 1], c_log2, -m_use));
      if (nb == 0) lsum0 += e0 + e1; else lsum1 += e0 + e1;
      const f32x2 two = {e0, e1};
      const bf16x2 b2 = __builtin_convertvector(two, bf16x2);
      p[nb][mb][r >> 3][r & 7] = b2[0];
      p[nb][mb][r >> 3][(r & 7) + 1] = b2[1];
    }
    // keep this round's adds in this round (they would otherwise sink to the end of the block)
    asm volatile("" : "+v"(lsum0), "+v"(lsum1));
    __builtin_amdgcn_sched_barrier(0);
  }
  st.l[0] += lsum0;
  st.l[1] += lsum1;
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

// has_ref (wave-uniform): whether the reference of the optimistic pass has been
// taken; the first computed step takes it.
template <int MB, int PASS>
__device__ inline void contiguous_step(WaveState &st, bool &has_ref, const LaneOfs &lo, const char *tK,
                                       const char *tV, int kbase, const MaskP &mp, float c_log2, int lane) {
  const int cls = classify_step<32 * MB>(kbase, mp);
  if (cls == 0) return;
  const bool first = PASS == PASS_OPT && !has_ref;
  has_ref = true;
  step_compute<MB, false, PASS>(st, lo, tK, tV, kbase, nullptr, mp, cls == 2 ? 1 : 0, first, c_log2, lane);
}

template <int MB, int PASS>
__device__ inline void gathered_step(WaveState &st, bool &has_ref, const LaneOfs &lo, const char *tK,
                                     const char *tV, const int *cols, const MaskP &mp, float c_log2, int lane) {
  const bool first = PASS == PASS_OPT && !has_ref;
  has_ref = true;
  step_compute<MB, true, PASS>(st, lo, tK, tV, 0, cols, mp, 1, first, c_log2, lane);
}

// After the optimistic pass: true (wave-uniform) if some row of the wave must be
// redone exactly: its sum overflowed (logits far above the reference), or it is
// zero or nearly so.  The latter happens to a row whose reference stayed at the
// neutral 0 (no permitted key in the wave's first step) or far above its own
// logits while all of them lie below about -100 in the base-2 domain: p then
// flushes to zero although the row is well defined under Eq. 1.  A row that
// really has no permitted key also takes the exact pass (and ends with zeros);
// only Vertical-Slash blocks before the first kept line have such rows.
__device__ inline bool needs_exact(const WaveState &st) {
  bool bad = false;
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    const float l = st.l[nb] + __shfl_xor(st.l[nb], 32);
    bad = bad || !(l < L_LIMIT) || l < L_TINY;
  }
  return __builtin_amdgcn_ballot_w64(bad) != 0;
}

// Exact scheme, pass 1 set-up: zero reference, st.l collects the row max.
__device__ inline void reset_for_max_pass(WaveState &st) {
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) { set_reference(st, nb, 0.f); st.l[nb] = -INFINITY; }
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.o[db][nb][r] = 0.f;
}

// Exact scheme, between the passes: the row max becomes the reference.
__device__ inline void finish_max_pass(WaveState &st, float c_log2) {
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    const float m = fmaxf(st.l[nb], __shfl_xor(st.l[nb], 32)) * c_log2;
    set_reference(st, nb, m == -INFINITY ? 0.f : m);
    st.l[nb] = 0.f;
  }
}

// ---------------------------------------------------------------------------
// A-shape (and dense causal: n_init = 0, n_local >= N).  4 waves, 256 query
// rows of one head per workgroup; shared 64-key K/V tiles.
// LDS: 3 K slots + 3 V slots of 16 KiB (the exact fallback pass uses 2 + 2).
// ---------------------------------------------------------------------------
struct AshapeCtx {
  const bf16_t *kh, *vh;
  int64_t k_st, v_st;
  DmaLane dk, dv;
  int N, T1, T, s2;
  char *lds;
  float c_log2;
  __device__ inline int tile_base(int t) const { return t < T1 ? t * BK : s2 + (t - T1) * BK; }
};

template <int PASS>
__device__ inline void ashape_pass(const AshapeCtx &c, WaveState &st, const LaneOfs &lo, const MaskP &mp,
                                   int wave, int lane) {
  auto fetch = [&](int t) {
    char *stg = c.lds + (t & 1) * 2 * TILE_BYTES;
    dma_rows<4, 64, true>(c.kh, c.k_st, c.dk, c.tile_base(t), nullptr, c.N, stg, wave, lane);
    dma_rows<4, 64, true>(c.vh, c.v_st, c.dv, c.tile_base(t), nullptr, c.N, stg + TILE_BYTES, wave, lane);
  };
  bool has_ref = false;
  fetch(0);
  MINF_WAIT_VMCNT(0);
  __syncthreads();
  for (int t = 0; t < c.T; ++t) {
    if (t + 1 < c.T) fetch(t + 1);
    const char *stg = c.lds + (t & 1) * 2 * TILE_BYTES;
    contiguous_step<2, PASS>(st, has_ref, lo, stg, stg + TILE_BYTES, c.tile_base(t), mp, c.c_log2, lane);
    MINF_WAIT_VMCNT(0);
    __syncthreads();
  }
}

// K Q^T MFMA with the accumulator in ordinary vector registers and the Q operand
// in accumulator registers.  The vector ALU cannot read accumulator registers
// directly, and v_accvgpr_read runs on the matrix pipeline (measured: it queues
// behind the MFMAs instead of overlapping them), so logits that the softmax is
// to consume while MFMAs run must be produced in vector registers.  The compiler
// picks one register class for all MFMA results of a kernel, hence assembly.
// Wait states the compiler cannot see: a result is read by the vector ALU only
// after at least four later MFMAs have issued (each occupies the pipeline for 8
// passes), and by an MFMA on the same accumulator only after three others.
typedef int i32x4 __attribute__((ext_vector_type(4)));
__device__ inline void mfma_qk_first(f32x16 &acc, bf16x8 k, const i32x4 &q) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0"
               : "=&v"(acc) : "a"(__builtin_bit_cast(i32x4, k)), "a"(q));
}
__device__ inline void mfma_qk_acc(f32x16 &acc, bf16x8 k, const i32x4 &q) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0"
               : "+v"(acc) : "a"(__builtin_bit_cast(i32x4, k)), "a"(q));
}

// Q operands of the pipelined pass, held in accumulator registers for the whole pass.
struct QAcc {
  i32x4 q[2][8];
};
__device__ inline void pin_q(QAcc &qa, const WaveState &st) {
#pragma unroll
  for (int nb = 0; nb < 2; ++nb)
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      qa.q[nb][ks] = __builtin_bit_cast(i32x4, st.q[nb][ks]);
      asm volatile("" : "+a"(qa.q[nb][ks]));
    }
}

// K Q^T of one tile into vector registers (start of the pipeline).
__device__ inline void qk_tile_v(f32x16 (&s)[2][2], const QAcc &qa, const LaneOfs &lo, const char *tK) {
#pragma unroll
  for (int ks = 0; ks < 8; ++ks)
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
      const bf16x8 a = lds_read_k(tK, lo.k[ks] + mb * HALF_BYTES);
      if (ks == 0) {
        mfma_qk_first(s[mb][0], a, qa.q[0][0]);
        mfma_qk_first(s[mb][1], a, qa.q[1][0]);
      } else {
        mfma_qk_acc(s[mb][0], a, qa.q[0][ks]);
        mfma_qk_acc(s[mb][1], a, qa.q[1][ks]);
      }
    }
  // the vector ALU may read s 18 wait states after the last MFMA was issued
  asm volatile("s_nop 15\n\ts_nop 3" ::: "memory");
}

// This wave's quarter of the fetch of a 64-row tile that lies wholly inside
// [0, N): rows 16w .. 16w+15, i.e. the 1 KiB blocks 4w .. 4w+3 of the tile in LDS.
// ROWS256: rows are 256 bytes apart in global memory as they are in LDS, so the
// four blocks are 1 KiB apart on both sides and one base pair and one M0 value
// serve all four loads through the instruction's immediate offset (it shifts the
// global and the LDS address alike).  Otherwise each block gets its own base.
struct WaveDma {
  unsigned k_voff[4], v_voff[4];   // per lane, block 4w + i
  unsigned k_rb, v_rb;             // bytes between rows
  const char *kw, *vw;             // head base + 16 w rows
  unsigned lds_w;                  // 4 w KiB
};
template <int I>
__device__ inline void dma16_imm(const char *ubase, unsigned voff, unsigned lds_addr) {
  if (I == 0) asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" :: "v"(voff), "s"(ubase), "s"(lds_addr) : "memory");
  if (I == 1) asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 offset:1024" :: "v"(voff), "s"(ubase), "s"(lds_addr) : "memory");
  if (I == 2) asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 offset:2048" :: "v"(voff), "s"(ubase), "s"(lds_addr) : "memory");
  if (I == 3) asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 offset:3072" :: "v"(voff), "s"(ubase), "s"(lds_addr) : "memory");
}
template <bool ROWS256, int I>
__device__ inline void dma_block(const char *tile_w, unsigned rb, unsigned voff, unsigned lds_tile_w) {
  if (ROWS256) dma16_imm<I>(tile_w, voff, lds_tile_w);
  else dma16_imm<0>(tile_w + (size_t)(4 * I) * rb, voff, lds_tile_w + I * 1024);
}

// Class of the 64-key tile at kb for the wave whose rows are q0 .. q0+63 under
// the A-shape mask, with the comparisons' constants taken out of the loop:
// 0 = nothing to attend, 1 = all attended, 2 = mixed.
struct AshapeCls {
  int qlast, n_init, a, b, c, d;
  __device__ inline void init(const MaskP &mp) {
    qlast = mp.q0 + BQ - 1; n_init = mp.n_init;
    a = mp.q0 - (BK - 1) - mp.n_local;   // kb <= a: the tile ends before the window of the first row starts
    b = mp.q0 - (BK - 1);                // kb <= b: the tile ends at or before the first row (no causal cut)
    c = mp.n_init - (BK - 1);            // kb <  c: the tile lies inside the sink
    d = qlast - mp.n_local;              // kb >  d: the tile starts inside the window of the last row
  }
  __device__ inline int of(int kb) const {
    if (kb > qlast || (kb >= n_init && kb <= a)) return 0;
    return (kb <= b && (kb < c || kb > d)) ? 1 : 2;
  }
};

// Optimistic pass of the shared-tile kernel, software pipelined three deep.
// Iteration t: the matrix cores alternate between the logits of tile t+1
// (K Q^T) and the output update of tile t-1 (V^T P^T) while the vector ALU turns
// the logits of tile t into P(t), so all exp / convert / row-sum work runs in
// the shadow of MFMAs that do not depend on it.  With one wave per SIMD the wave
// issues at most one instruction every four cycles, so the iteration is built
// to a budget of instructions: about 9 per MFMA all told.
//  - One iteration = 8 rounds x 4 groups; a group is 2 MFMAs and 2 logits of the
//    softmax.  The LDS reads of a round's operands are issued as one batch at
//    the top of the round before (one wait per round); the wave's 8 tile loads
//    go out one per round (back to back they stall the wave until the memory
//    pipeline has taken them); scalar bookkeeping sits between the rounds' MFMAs.
//  - K and V each cycle through four LDS slots of which three hold live tiles;
//    iteration t issues the loads of K(t+3) and V(t+1) in its rounds 4..7 and
//    reads K(t+1) and V(t-1).  Slot of tile i: i mod 4; the loop is unrolled four
//    times, so every slot address is an immediate.  Past the last tile the loads
//    repeat it into the free slot, so that every iteration issues 8 loads.
//  - The one barrier of an iteration sits after round 3 (with a wait for the
//    loads of the iteration before).  The tiles the next iteration reads are
//    therefore confirmed half an iteration early, and its first operands are
//    fetched from LDS in round 7: no LDS latency is exposed at the top of an
//    iteration and nothing but the loop branch separates two iterations.
//  - Every wave runs every iteration on every tile of the workgroup's key range,
//    also on tiles outside its own rows' mask (the four waves meet at a barrier
//    each iteration, so skipping would only idle): such a tile gets P = 0 via an
//    infinite reference.  The body is one straight path, which keeps the 128
//    output accumulators in place; the first iteration multiplies a zero P(-1)
//    with V(0), the last two form logits nobody consumes.
template <bool ROWS256>
struct AshapeLoop {
  WaveState &st;
  const QAcc &qa;
  const LaneOfs &lo;
  const MaskP &mp;
  const WaveDma &d;
  AshapeCls cls;
  float c_log2;
  int lane;
  int T, T1, s2;
  // K slots at lds + i * 16 KiB, V slots at lds + (4 + i) * 16 KiB, i < 4: tile s lives in slot
  // s mod 4.  Three tiles of each kind are live at a time; the fourth slot makes the ring length a
  // power of two, so that the loop, unrolled four times, has every slot as a compile-time constant
  // (with the slot offset in a register every LDS operand read cost an address add: 51 of the
  // about 1100 instructions of an iteration).
  char *lds;
  static constexpr unsigned k_slot(int i) { return (unsigned)(i & 3) * TILE_BYTES; }
  static constexpr unsigned v_slot(int i) { return (unsigned)(4 + (i & 3)) * TILE_BYTES; }
  int kb1, kb2, kb3, ti3;    // key bases of tiles t+1, t+2, t+3 (indices clamped to T-1); index of the last
  int cls_cur;
  bool has_ref;

  // scalar operands of the coming iteration
  const char *kt_, *vt_;
  int cls_nxt_;

  __device__ inline int tile_base(int i) const { return i < T1 ? i * BK : s2 + (i - T1) * BK; }

  // for iteration t, from the tile state of iteration t
  __device__ inline void prepare(int t) {
    kt_ = d.kw + (size_t)kb3 * d.k_rb;                                  // K(t+3) -> slot (t+3) mod 4
    vt_ = d.vw + (size_t)kb1 * d.v_rb;                                  // V(t+1) -> slot (t+1) mod 4
    cls_nxt_ = t + 1 < T ? cls.of(kb1) : 0;
  }

  template <int I>
  __device__ inline void load_k(int kb, unsigned slot_ofs) const {
    dma_block<ROWS256, I>(d.kw + (size_t)kb * d.k_rb, d.k_rb, d.k_voff[I], lds_addr_of(lds) + slot_ofs + d.lds_w);
  }
  template <int I>
  __device__ inline void load_v(int kb, unsigned slot_ofs) const {
    dma_block<ROWS256, I>(d.vw + (size_t)kb * d.v_rb, d.v_rb, d.v_voff[I],
                          lds_addr_of(lds) + 4 * TILE_BYTES + slot_ofs + d.lds_w);
  }
  // first operands of an iteration (k-step 0 of both key blocks, output update steps 0, 1): read
  // during the last round of the iteration before
  struct Lead {
    bf16x8 k[2], v[2];
  };
  // for the iteration of phase PH: K(t+1) and V(t-1) (V(0) in the very first one: zero P(-1))
  template <int PH, bool FIRST>
  __device__ inline void read_lead(Lead &ld) const {
    const char *tK = lds + k_slot(PH + 1), *tV = lds + v_slot(FIRST ? 0 : PH + 3);
    ld.k[0] = lds_read_k(tK, lo.k[0]);
    ld.k[1] = lds_read_k(tK, lo.k[0] + HALF_BYTES);
    ld.v[0] = lds_read_vt(tV, lo.v[0][0], lo.v[0][1]);
    ld.v[1] = lds_read_vt(tV, lo.v[1][0], lo.v[1][1]);
  }

  // Iteration t, PH = t mod 4.
  template <int PH, bool FIRST>
  __device__ inline void iter(int t, f32x16 (&s_cur)[2][2], f32x16 (&s_nxt)[2][2], bf16x8 (&p_prev)[2][2][2],
                              bf16x8 (&p_cur)[2][2][2], Lead &lead) {
    const char *tK = lds + k_slot(PH + 1), *tV = lds + v_slot(FIRST ? 0 : PH + 3);
    auto fetch_v = [&](int i) {            // PV step i = (mb, t, db)
      const int mb = i / 8, tt = (i / 4) & 1, db = i & 3;
      const int base = (32 * mb + 16 * tt) * ROW_BYTES;
      return lds_read_vt(tV, lo.v[db][0] + base, lo.v[db][1] + base);
    };
    bf16x8 kf[8][2], vf[16];
    kf[0][0] = lead.k[0];
    kf[0][1] = lead.k[1];
    vf[0] = lead.v[0];
    vf[1] = lead.v[1];
    // the iteration's scalar operands were prepared during the previous one
    const char *kt = kt_, *vt = vt_;
    const unsigned k_dst = lds_addr_of(lds) + k_slot(PH + 3) + d.lds_w;
    const unsigned v_dst = lds_addr_of(lds) + v_slot(PH + 1) + d.lds_w;
    const int cls_nxt = cls_nxt_, kb_nxt = kb1;
    const bool attend_cur = cls_cur != 0;
    // ... and the next one's are prepared in round 5, between MFMAs
    auto prepare_next = [&]() {
      kb1 = kb2; kb2 = kb3;
      if (ti3 + 1 < T) {
        ++ti3;
        kb3 = ti3 == T1 ? s2 : kb3 + BK;
      }
      prepare(t + 1);
    };
    // a tile this wave must not attend at all gets an infinite reference: P = exp2(-inf) = 0
    const float m0 = attend_cur ? st.m[0] : INFINITY, m1 = attend_cur ? st.m[1] : INFINITY;
    float lsum0 = 0.f, lsum1 = 0.f;
    // Logits are walked so that round 2j + nb turns the 8 logits per lane of key
    // group j = (mb, t) and query block nb into one B operand of the output
    // update: P(t) group j is born in the rounds in which P(t-1) group j is last
    // used, so the two generations of P share registers (about 40 instead of 64).
    // Pair e (even) of the 64 logits per lane: exponentials first; sum and conversion follow one
    // pair later, so that no instruction consumes a transcendental result right behind it.
    float pe0 = 0.f, pe1 = 0.f, ne0 = 0.f, ne1 = 0.f;
    auto exp_pair = [&](int e) {
      const int j = e / 16, nb = (e / 8) & 1, mb = j / 2, r = 8 * (j & 1) + (e & 7);
      const float m_use = nb == 0 ? m0 : m1;
      ne0 = fast_exp2(fmaf(s_cur[mb][nb][r], c_log2, -m_use));
      ne1 = fast_exp2(fmaf(s_cur[mb][nb][r + 1], c_log2, -m_use));
      asm volatile("" : "+v"(ne0), "+v"(ne1));
    };
    auto finish_pair = [&](int e) {        // pair e's exponentials are in pe0, pe1
      const int j = e / 16, nb = (e / 8) & 1, mb = j / 2, r = 8 * (j & 1) + (e & 7);
      if (nb == 0) lsum0 += pe0 + pe1; else lsum1 += pe0 + pe1;
      const f32x2 two = {pe0, pe1};
      unsigned pk = __builtin_bit_cast(unsigned, __builtin_convertvector(two, bf16x2));
      asm volatile("" : "+v"(pk), "+v"(lsum0), "+v"(lsum1));   // convert here, not where P is consumed
      const bf16x2 b2 = __builtin_bit_cast(bf16x2, pk);
      p_cur[nb][mb][r >> 3][r & 7] = b2[0];
      p_cur[nb][mb][r >> 3][(r & 7) + 1] = b2[1];
    };
    auto sum_pair = [&](int e) {           // finishes pair e - 2, then pair e's exponentials take its place
      if (e > 0) finish_pair(e - 2);
      pe0 = ne0; pe1 = ne1;
    };
    // One round = 8 groups, each opened by ONE MFMA: the wave issues in order, and a second MFMA
    // right behind the first stalls the issue for the 32 cycles the first occupies the pipeline.
    auto round = [&](auto rc_) {
      constexpr int r = decltype(rc_)::value;
      // the operands of this round went out during the previous one
      __builtin_amdgcn_s_waitcnt(0xC07F);
      // groups 0..3: logits of key blocks 0, 1 (k-step r) for query blocks 0, 1
      if (r == 0) mfma_qk_first(s_nxt[0][0], kf[0][0], qa.q[0][0]);
      else mfma_qk_acc(s_nxt[0][0], kf[r][0], qa.q[0][r]);
      exp_pair(8 * r);
      if (r + 1 < 8) {
        kf[(r + 1) & 7][0] = lds_read_k(tK, lo.k[(r + 1) & 7]);
        kf[(r + 1) & 7][1] = lds_read_k(tK, lo.k[(r + 1) & 7] + HALF_BYTES);
      }
      __builtin_amdgcn_sched_barrier(0);
      if (r == 0) mfma_qk_first(s_nxt[0][1], kf[0][0], qa.q[1][0]);
      else mfma_qk_acc(s_nxt[0][1], kf[r][0], qa.q[1][r]);
      sum_pair(8 * r);
      if (r >= 4) dma_block<ROWS256, r & 3>(kt, d.k_rb, d.k_voff[r & 3], k_dst);
      __builtin_amdgcn_sched_barrier(0);
      if (r == 0) mfma_qk_first(s_nxt[1][0], kf[0][1], qa.q[0][0]);
      else mfma_qk_acc(s_nxt[1][0], kf[r][1], qa.q[0][r]);
      exp_pair(8 * r + 2);
      if (r + 1 < 8) {
        vf[(2 * r + 2) & 15] = fetch_v((2 * r + 2) & 15);
        vf[(2 * r + 3) & 15] = fetch_v((2 * r + 3) & 15);
      }
      __builtin_amdgcn_sched_barrier(0);
      if (r == 0) mfma_qk_first(s_nxt[1][1], kf[0][1], qa.q[1][0]);
      else mfma_qk_acc(s_nxt[1][1], kf[r][1], qa.q[1][r]);
      sum_pair(8 * r + 2);
      if (r >= 4) dma_block<ROWS256, r & 3>(vt, d.v_rb, d.v_voff[r & 3], v_dst);
      if (r == 5) prepare_next();
      __builtin_amdgcn_sched_barrier(0);
      // groups 4..7: output update steps 2r, 2r + 1 of the previous tile
#pragma unroll
      for (int g = 0; g < 2; ++g) {
        const int i = 2 * r + g;
        const int mb = i / 8, tt = (i / 4) & 1, db = i & 3;
        st.o[db][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i], p_prev[0][mb][tt], st.o[db][0], 0, 0, 0);
        exp_pair(8 * r + 4 + 2 * g);
        __builtin_amdgcn_sched_barrier(0);
        st.o[db][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i], p_prev[1][mb][tt], st.o[db][1], 0, 0, 0);
        sum_pair(8 * r + 4 + 2 * g);
        if (r == 7 && g == 1) finish_pair(62);
        // the first operands of the next iteration (its tiles were confirmed at this iteration's barrier)
        if (r == 7 && g == 0) read_lead<(PH + 1) & 3, false>(lead);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (r == 3) {
        // The iteration's one barrier sits in its middle.  Landed and visible behind it: the loads
        // issued in rounds 4..7 of the iteration before, K(t+2) and V(t), which the next iteration
        // reads.  Free behind it: the slots this iteration's loads (rounds 4..7) overwrite, which
        // held K(t-1) and V(t-3), last read two and three iterations ago.
        MINF_WAIT_VMCNT(0);
        __syncthreads();
      }
    };
    round(std::integral_constant<int, 0>{});
    round(std::integral_constant<int, 1>{});
    round(std::integral_constant<int, 2>{});
    round(std::integral_constant<int, 3>{});
    round(std::integral_constant<int, 4>{});
    round(std::integral_constant<int, 5>{});
    round(std::integral_constant<int, 6>{});
    round(std::integral_constant<int, 7>{});
    if (attend_cur) {
      st.l[0] += lsum0;
      st.l[1] += lsum1;
    }
    // logits of tile t+1: element mask and / or the exponent reference (rare)
    if (cls_nxt == 2 || (cls_nxt != 0 && !has_ref)) {
      special_tile<2>(s_nxt, st, kb_nxt, mp, cls_nxt == 2, !has_ref, c_log2, lane);
      has_ref = true;
    }
    cls_cur = cls_nxt;
  }
};

template <bool ROWS256>
__device__ inline void ashape_pass_pipelined(const AshapeCtx &c, const WaveDma &d, WaveState &st,
                                             const LaneOfs &lo, const MaskP &mp, int lane) {
  QAcc qa;
  pin_q(qa, st);
  AshapeLoop<ROWS256> lp{st, qa, lo, mp, d};
  lp.cls.init(mp);
  lp.c_log2 = c.c_log2; lp.lane = lane; lp.T = c.T; lp.T1 = c.T1; lp.s2 = c.s2; lp.lds = c.lds;
  lp.has_ref = false;
  const int last = c.T - 1;
  const int kb0 = lp.tile_base(0);
  lp.kb1 = lp.tile_base(min(1, last)); lp.kb2 = lp.tile_base(min(2, last));
  lp.ti3 = min(3, last); lp.kb3 = lp.tile_base(lp.ti3);
  f32x16 sa[2][2], sb[2][2];
  bf16x8 pa[2][2][2], pb[2][2][2];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) (&pa[0][0][0])[i][j] = (__bf16)0.f;
  // K(0), K(1), K(2) into K slots 0, 1, 2 and V(0) into V slot 0
  lp.template load_k<0>(kb0, 0); lp.template load_k<1>(kb0, 0); lp.template load_k<2>(kb0, 0); lp.template load_k<3>(kb0, 0);
  lp.template load_k<0>(lp.kb1, TILE_BYTES); lp.template load_k<1>(lp.kb1, TILE_BYTES);
  lp.template load_k<2>(lp.kb1, TILE_BYTES); lp.template load_k<3>(lp.kb1, TILE_BYTES);
  lp.template load_k<0>(lp.kb2, 2 * TILE_BYTES); lp.template load_k<1>(lp.kb2, 2 * TILE_BYTES);
  lp.template load_k<2>(lp.kb2, 2 * TILE_BYTES); lp.template load_k<3>(lp.kb2, 2 * TILE_BYTES);
  lp.template load_v<0>(kb0, 0); lp.template load_v<1>(kb0, 0); lp.template load_v<2>(kb0, 0); lp.template load_v<3>(kb0, 0);
  MINF_WAIT_VMCNT(0);
  __syncthreads();
  lp.cls_cur = lp.cls.of(kb0);
  // also for a tile this wave does not attend: its (finite) logits are turned into P = 0
  qk_tile_v(sa, qa, lo, c.lds);
  if (lp.cls_cur != 0) {
    special_tile<2>(sa, st, kb0, mp, lp.cls_cur == 2, true, c.c_log2, lane);
    lp.has_ref = true;
  }
  __syncthreads();   // all waves are done with K(0) before iteration 0 overwrites it with K(3)
  lp.prepare(0);
  typename AshapeLoop<ROWS256>::Lead lead;
  lp.template read_lead<0, true>(lead);
  // iterations t = 0 .. T (the last one finishes the output update of tile T-1); T is the same
  // for the four waves, which meet at the barrier of every iteration
  lp.template iter<0, true>(0, sa, sb, pa, pb, lead);
  for (int t = 1; t <= c.T;) {
    lp.template iter<1, false>(t, sb, sa, pb, pa, lead);
    if (++t > c.T) break;
    lp.template iter<2, false>(t, sa, sb, pa, pb, lead);
    if (++t > c.T) break;
    lp.template iter<3, false>(t, sb, sa, pb, pa, lead);
    if (++t > c.T) break;
    lp.template iter<0, false>(t, sa, sb, pa, pb, lead);
    ++t;
  }
  MINF_WAIT_VMCNT(0);   // the repeated loads of the last iterations
  __syncthreads();
}

template <bool ROWS256>
__global__ __launch_bounds__(256) void ashape_kernel(QKV x, HeadList hl, int n_init, int n_local,
                                                     Sched sched) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int NB = x.N / BQ;
  int slot, sb;
  if (!decode_wg(sched, slot, sb)) return;
  const int head = __builtin_amdgcn_readfirstlane(hl.h[slot]);
  const int kvh = to_sgpr(head / x.group);
  const bf16_t *qh = x.q + head * x.q_sh;
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
  AshapeCtx c;
  c.kh = x.k + kvh * x.k_sh; c.vh = x.v + kvh * x.v_sh; c.k_st = x.k_st; c.v_st = x.v_st;
  c.N = x.N; c.T1 = e1 / BK; c.T = c.T1 + (wq1 - s2) / BK; c.s2 = s2; c.lds = lds; c.c_log2 = x.c_log2;
  dma_lane_init(c.dk, x.k_st, lane);
  dma_lane_init(c.dv, x.v_st, lane);
  WaveDma d;
#pragma unroll
  for (int i = 0; i < 4; ++i) { d.k_voff[i] = c.dk.voff[i]; d.v_voff[i] = c.dv.voff[i]; }
  d.k_rb = (unsigned)x.k_st * 2u; d.v_rb = (unsigned)x.v_st * 2u;
  d.kw = reinterpret_cast<const char *>(c.kh) + (size_t)(16 * wave) * d.k_rb;
  d.vw = reinterpret_cast<const char *>(c.vh) + (size_t)(16 * wave) * d.v_rb;
  d.lds_w = wave * 4096;

  ashape_pass_pipelined<ROWS256>(c, d, st, lo, mp, lane);
  if (__syncthreads_or(needs_exact(st) ? 1 : 0)) {
    load_q(st, qh, x.q_st, q0, lane);   // the pipelined pass kept Q in accumulator registers only
    reset_for_max_pass(st);
    ashape_pass<PASS_MAX>(c, st, lo, mp, wave, lane);
    finish_max_pass(st, x.c_log2);
    ashape_pass<PASS_FIX>(c, st, lo, mp, wave, lane);
  }
  if (active) wave_finish(st, oh, x.o_st, q0, lds + wave * TILE_BYTES, lane);
}

// Makes LDS writes of this wave's lanes visible to its other lanes.  LDS operations of one wave
// execute in issue order; the fences only keep the compiler from reordering them.  (The column
// lists of the Vertical-Slash kernels are private to a wave, and the waves of a workgroup walk
// lists of different lengths, so no workgroup barrier may be used there.)
__device__ inline void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---------------------------------------------------------------------------
// Single-wave kernels: 32-key steps through private rings.
// LDS: 2 K slots + 3 V slots of 8 KiB = 40 KiB (the column list of the
// Vertical-Slash gather phase lives in the third V slot).
// One step = 16 global_load_lds instructions (8 K + 8 V); the wave keeps the
// next steps' loads in flight while it computes the current one.
// ---------------------------------------------------------------------------
// Per-wave LDS ring of the single-wave kernels: K slots 0, 1, then V slots 0, 1, 2 (8 KiB each,
// 40 KiB: four workgroups fill a CU's 160 KiB).  The two-deep pipelines use V slots 0 and 1.
struct StepBuf {
  char *lds;
  __device__ inline char *k(int s) const { return lds + s * HALF_BYTES; }
  __device__ inline char *v(int s) const { return lds + (2 + s) * HALF_BYTES; }
};

template <bool CONTIG, class Buf>
__device__ inline void fetch_step(const Buf &sb, int s, const bf16_t *kh, const bf16_t *vh, int64_t k_st,
                                  int64_t v_st, int kbase, const int *cols, int N, int lane) {
  DmaLane dk, dv;
  dma_lane_init(dk, k_st, lane);
  dma_lane_init(dv, v_st, lane);
  dma_rows<1, 32, CONTIG>(kh, k_st, dk, kbase, cols, N, sb.k(s), 0, lane);
  dma_rows<1, 32, CONTIG>(vh, v_st, dv, kbase, cols, N, sb.v(s), 0, lane);
}

// Rare path on fresh logits of a gathered step: attended iff key <= query row.
__device__ inline void special_gather(f32x16 (&s)[1][2], WaveState &st, const int *cols, const MaskP &mp,
                                      bool first, float c_log2, int lane) {
  const int n = lane & 31, h = lane >> 5;
  int keys[16];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int4 a = *reinterpret_cast<const int4 *>(cols + 16 * t + 8 * h);
    const int4 b = *reinterpret_cast<const int4 *>(cols + 16 * t + 8 * h + 4);
    keys[8 * t + 0] = a.x; keys[8 * t + 1] = a.y; keys[8 * t + 2] = a.z; keys[8 * t + 3] = a.w;
    keys[8 * t + 4] = b.x; keys[8 * t + 5] = b.y; keys[8 * t + 6] = b.z; keys[8 * t + 7] = b.w;
  }
#pragma unroll
  for (int r = 0; r < 16; ++r)
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) s[0][nb][r] = keys[r] <= mp.q0 + 32 * nb + n ? s[0][nb][r] : -INFINITY;
  if (first) {
    MaskP none = mp;
    special_tile<1>(s, st, 0, none, false, true, c_log2, lane);
  }
}

// One 32-key step of a single-wave kernel.  cols == nullptr: keys kbase .. kbase+31
// with the mask window [lo, hi); else keys cols[0..31] (LDS).  cls 1: no element is
// masked, 2: the element mask must be applied.
struct Step {
  int kbase, lo, hi, cls;
  const int *cols;
};

// Two loads of one round of the single-wave pipeline: blocks B and B + 1 of the
// eight 1 KiB blocks of a 32-row step, both with the M0 value set here.
// ROWS256 (rows 256 bytes apart in global memory, as in LDS): blocks 0..3 hang off
// base and M0 through the immediate offset, blocks 4..7 off base + 4096.
template <bool ROWS256, int B>
__device__ inline void dma_pair(const char *step_row0, unsigned rb, const unsigned (&voff)[4], unsigned lds_step) {
  if (ROWS256) {
    const char *base = step_row0 + (B >= 4 ? 4096 : 0);
    const unsigned m = lds_step + (B >= 4 ? 4096 : 0);
    if ((B & 3) == 0)
      asm volatile("s_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %2\n\t"
                   "global_load_lds_dwordx4 %1, %2 offset:1024"
                   :: "v"(voff[0]), "v"(voff[1]), "s"(base), "s"(m) : "memory");
    else
      asm volatile("s_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %2 offset:2048\n\t"
                   "global_load_lds_dwordx4 %1, %2 offset:3072"
                   :: "v"(voff[2]), "v"(voff[3]), "s"(base), "s"(m) : "memory");
  } else {
    dma16_imm<0>(step_row0 + (size_t)(4 * B) * rb, voff[B & 3], lds_step + B * 1024);
    dma16_imm<0>(step_row0 + (size_t)(4 * B + 4) * rb, voff[(B + 1) & 3], lds_step + (B + 1) * 1024);
  }
}
// Gathered rows: lane L of block blk fetches chunk c of row cols[4 blk + L / 16];
// the byte offset key * rb + 16 c fits 32 bits (checked on the host: N rb < 2^32),
// key < 2^24.  KEY_NONE entries read the last row (the caller masks them): one unsigned minimum
// with N - 1 instead of a compare and a select.
template <int B>
__device__ inline void dma_pair_gather(const char *head, unsigned rb, const int *cols, unsigned lds_step,
                                       int lane, unsigned last_row) {
  const int rl = lane >> 4, cpos = lane & 15;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int blk = B + j, r = 4 * blk + rl;
    const unsigned key = min((unsigned)cols[r], last_row);
    const unsigned ofs = __umul24(key, rb) + (unsigned)((cpos ^ swz_f(r)) << 4);
    dma16_su(head, ofs, lds_step + blk * 1024);
  }
}

// Software-pipelined optimistic pass over the 32-key steps a generator yields
// (skipped steps are never yielded), one wave, private K/V double buffers.
// Iteration t: the logits of step t+1 (K Q^T, 16 MFMAs) are formed while the
// vector ALU turns the logits of step t into P(t); the output update of step t
// (16 MFMAs) follows its half of P(t) by three rounds.  Logits live in vector
// registers, Q and the LDS operands in accumulator registers (see mfma_qk_*).
// The iteration is built to an instruction budget like the shared-tile loop:
// 8 rounds; per round one batch of LDS reads for the round after and one wait;
// the 16 tile loads (K of step t+2 into the buffer step t's logits came from,
// V of step t+1 into the buffer of step t-1) go out two per round, K first: K
// must have landed at the top of the next iteration, V only by its round 2; the
// generator advances between MFMAs.  When the generator runs dry the loads
// repeat an earlier step into the free buffer and the MFMAs form logits nobody
// consumes, so that the body stays one straight path.
template <class Gen, bool GATHER, bool ROWS256>
struct WavePipe {
  Gen &gen;
  WaveState &st;
  const QAcc &qa;
  bool &has_ref;
  const LaneOfs &lo;
  StepBuf buf;
  const char *kh, *vh;       // head bases (bytes)
  unsigned k_rb, v_rb;
  const DmaLane &dk, &dv;
  int N;
  MaskP mp;
  float c_log2;
  int lane;
  Step d0, d1, d2;          // steps t, t+1, t+2
  bool h0, h1, h2;

  __device__ inline const char *row0(const char *head, unsigned rb, const Step &d) const {
    // the generators yield steps inside [0, N); step descriptors come out of LDS lists or lanes,
    // i.e. out of vector registers, although they are wave-uniform
    const unsigned kb = (unsigned)__builtin_amdgcn_readfirstlane(d.kbase);
    return head + (uint64_t)kb * rb;
  }
  template <int R>
  __device__ inline void round_dma(const char *kt, const char *vt, const int *kcols, const int *vcols,
                                   unsigned k_dst, unsigned v_dst) const {
    // K in rounds 0..3, V in rounds 4..7: K is needed at the top of the next iteration, V not
    // before its round 2
    constexpr bool k_now = R < 4;
    if (GATHER) {
      if (k_now) dma_pair_gather<2 * (R & 3)>(kh, k_rb, kcols, k_dst, lane, (unsigned)N - 1u);
      else dma_pair_gather<2 * (R & 3)>(vh, v_rb, vcols, v_dst, lane, (unsigned)N - 1u);
    } else {
      if (k_now) dma_pair<ROWS256, 2 * (R & 3)>(kt, k_rb, dk.voff, k_dst);
      else dma_pair<ROWS256, 2 * (R & 3)>(vt, v_rb, dv.voff, v_dst);
    }
  }
  __device__ inline void fresh(f32x16 (&s)[1][2], const Step &d) {
    if (d.cls == 2 || !has_ref) {
      if (GATHER) {
        special_gather(s, st, d.cols, mp, !has_ref, c_log2, lane);
      } else {
        MaskP m = mp;
        m.lo = d.lo; m.hi = d.hi;
        if (d.cls == 2) window_mask<1>(s, d.kbase, m, lane);
        if (!has_ref) special_tile<1>(s, st, d.kbase, m, false, true, c_log2, lane);
      }
    }
    has_ref = true;
  }
  // K Q^T of one step into vector registers (start of the pipeline)
  __device__ inline void qk_first(f32x16 (&s)[1][2], const char *tK) const {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const bf16x8 a = lds_read_k(tK, lo.k[ks]);
      if (ks == 0) {
        mfma_qk_first(s[0][0], a, qa.q[0][0]);
        mfma_qk_first(s[0][1], a, qa.q[1][0]);
      } else {
        mfma_qk_acc(s[0][0], a, qa.q[0][ks]);
        mfma_qk_acc(s[0][1], a, qa.q[1][ks]);
      }
    }
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 7" ::: "memory");   // results readable by the vector ALU
  }

  __device__ inline void iter(int t, f32x16 (&s_cur)[1][2], f32x16 (&s_nxt)[1][2]) {
    MINF_WAIT_VMCNT(8);      // K of step t+1 has landed (V of step t, issued after it, may be in flight)
    const char *tK = buf.k((t + 1) & 1), *tV = buf.v(t & 1);
    const unsigned k_dst = lds_addr_of(buf.k(t & 1)), v_dst = lds_addr_of(buf.v((t + 1) & 1));
    bf16x8 kf[8], vf[8], p[2][2];
    kf[0] = lds_read_k(tK, lo.k[0]);
    const char *kt = row0(kh, k_rb, d2), *vt = row0(vh, v_rb, d1);
    const int *kcols = d2.cols, *vcols = d1.cols;     // the generator advances mid-iteration
    const float m0 = st.m[0], m1 = st.m[1];
    float lsum0 = 0.f, lsum1 = 0.f;
    auto fetch_v = [&](int i) {            // output update step i = (t, db)
      const int base = 16 * (i >> 2) * ROW_BYTES, db = i & 3;
      return lds_read_vt(tV, lo.v[db][0] + base, lo.v[db][1] + base);
    };
    // pair e of the 16 logit pairs per lane, walked [t][nb][r]: P group (nb, t) is
    // complete after pairs 8t + 4nb .. + 3.  The exponentials of pair e are issued
    // first, the sum and the conversion of pair e - 1 behind them: a transcendental
    // result is not consumed by the instruction right after it (no wait state).
    float pe0 = 0.f, pe1 = 0.f;
    auto finish_pair = [&](int e) {        // pair e's exponentials are in pe0, pe1
      const int tt = e >> 3, nb = (e >> 2) & 1;
      if (nb == 0) lsum0 += pe0 + pe1; else lsum1 += pe0 + pe1;
      const f32x2 two = {pe0, pe1};
      unsigned pk = __builtin_bit_cast(unsigned, __builtin_convertvector(two, bf16x2));
      asm volatile("" : "+v"(pk), "+v"(lsum0), "+v"(lsum1));
      const bf16x2 b2 = __builtin_bit_cast(bf16x2, pk);
      p[nb][tt][2 * (e & 3)] = b2[0];
      p[nb][tt][2 * (e & 3) + 1] = b2[1];
    };
    auto softmax2 = [&](int e) {
      const int tt = e >> 3, nb = (e >> 2) & 1, r = 8 * tt + 2 * (e & 3);
      const float m_use = nb == 0 ? m0 : m1;
      float e0 = fast_exp2(fmaf(s_cur[0][nb][r], c_log2, -m_use));
      float e1 = fast_exp2(fmaf(s_cur[0][nb][r + 1], c_log2, -m_use));
      asm volatile("" : "+v"(e0), "+v"(e1));
      if (e > 0) finish_pair(e - 1);
      pe0 = e0; pe1 = e1;
    };
    auto pv_step = [&](int i) {
      const int tt = i >> 2, db = i & 3;
      st.o[db][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i], p[0][tt], st.o[db][0], 0, 0, 0);
      st.o[db][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i], p[1][tt], st.o[db][1], 0, 0, 0);
    };
    // schedule per round: logit pairs [SM0, SM1) and output update steps [PV0, PV1)
    //  round        0  1  2  3  4  5  6  7
    //  pairs        3  3  2  3  3  2  -  -      (first half of P complete after round 2, second after 5)
    //  update steps -  -  -  1  2  1  2  2
    auto round = [&](auto rc_, auto sm0_, auto sm1_, auto pv0_, auto pv1_) {
      constexpr int r = decltype(rc_)::value, SM0 = decltype(sm0_)::value, SM1 = decltype(sm1_)::value;
      constexpr int PV0 = decltype(pv0_)::value, PV1 = decltype(pv1_)::value;
      // operands of the round after this one; then wait for this round's (issued a round ago)
      constexpr int NPV_NEXT = r == 2 ? 1 : r == 3 ? 2 : r == 4 ? 1 : (r == 5 || r == 6) ? 2 : 0;
      constexpr int PV_NEXT0 = PV1;
      if (r + 1 < 8) kf[(r + 1) & 7] = lds_read_k(tK, lo.k[(r + 1) & 7]);
#pragma unroll
      for (int i = 0; i < NPV_NEXT; ++i) vf[(PV_NEXT0 + i) & 7] = fetch_v((PV_NEXT0 + i) & 7);
      constexpr int NEW = (r + 1 < 8 ? 1 : 0) + 2 * NPV_NEXT;      // LDS reads just issued
      __builtin_amdgcn_s_waitcnt(0xC07F | (NEW << 8));
      round_dma<r>(kt, vt, kcols, vcols, k_dst, v_dst);
      if (r == 1) MINF_WAIT_VMCNT(4);      // V of step t has landed: round 2 starts reading it
      if (r == 0) {
        mfma_qk_first(s_nxt[0][0], kf[0], qa.q[0][0]);
        mfma_qk_first(s_nxt[0][1], kf[0], qa.q[1][0]);
      } else {
        mfma_qk_acc(s_nxt[0][0], kf[r], qa.q[0][r]);
        mfma_qk_acc(s_nxt[0][1], kf[r], qa.q[1][r]);
      }
#pragma unroll
      for (int e = SM0; e < SM1; ++e) {
        softmax2(e);
        if (e == 15) finish_pair(15);
        if (e + 1 < SM1 || PV0 == PV1) __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int i = PV0; i < PV1; ++i) {
        pv_step(i);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (r == 3) {
        // advance the generator between MFMAs: the step after d2
        d0 = d1; d1 = d2;
        h0 = h1; h1 = h2;
        Step dn = d2;
        h2 = h2 && gen.next(dn);
        if (h2) d2 = dn;
      }
      __builtin_amdgcn_sched_barrier(0);
    };
#define MINF_IC(n) std::integral_constant<int, n>{}
    round(MINF_IC(0), MINF_IC(0), MINF_IC(3), MINF_IC(0), MINF_IC(0));
    round(MINF_IC(1), MINF_IC(3), MINF_IC(6), MINF_IC(0), MINF_IC(0));
    round(MINF_IC(2), MINF_IC(6), MINF_IC(8), MINF_IC(0), MINF_IC(0));
    round(MINF_IC(3), MINF_IC(8), MINF_IC(11), MINF_IC(0), MINF_IC(1));
    round(MINF_IC(4), MINF_IC(11), MINF_IC(14), MINF_IC(1), MINF_IC(3));
    round(MINF_IC(5), MINF_IC(14), MINF_IC(16), MINF_IC(3), MINF_IC(4));
    round(MINF_IC(6), MINF_IC(16), MINF_IC(16), MINF_IC(4), MINF_IC(6));
    round(MINF_IC(7), MINF_IC(16), MINF_IC(16), MINF_IC(6), MINF_IC(8));
#undef MINF_IC
    st.l[0] += lsum0;
    st.l[1] += lsum1;
    // after the generator advanced in round 3: d0 = the step whose logits are now in s_nxt
    if (h0) fresh(s_nxt, d0);
  }
  template <bool IS_K>
  __device__ inline void fetch_whole(const Step &d, unsigned dst) const {
    const char *head = IS_K ? kh : vh;
    const unsigned rb = IS_K ? k_rb : v_rb;
    if (GATHER) {
      const unsigned last = (unsigned)N - 1u;
      dma_pair_gather<0>(head, rb, d.cols, dst, lane, last); dma_pair_gather<2>(head, rb, d.cols, dst, lane, last);
      dma_pair_gather<4>(head, rb, d.cols, dst, lane, last); dma_pair_gather<6>(head, rb, d.cols, dst, lane, last);
    } else {
      const char *a = row0(head, rb, d);
      const unsigned (&vo)[4] = IS_K ? dk.voff : dv.voff;
      dma_pair<ROWS256, 0>(a, rb, vo, dst); dma_pair<ROWS256, 2>(a, rb, vo, dst);
      dma_pair<ROWS256, 4>(a, rb, vo, dst); dma_pair<ROWS256, 6>(a, rb, vo, dst);
    }
  }
  __device__ inline void run() {
    h0 = gen.next(d0);
    if (!h0) return;
    d1 = d0;
    h1 = gen.next(d1);
    d2 = d1;
    h2 = h1 && gen.next(d2);
    // K of steps 0, 1 into K slots 0, 1, V of step 0 into V slot 0
    fetch_whole<true>(d0, lds_addr_of(buf.k(0)));
    fetch_whole<true>(d1, lds_addr_of(buf.k(1)));
    fetch_whole<false>(d0, lds_addr_of(buf.v(0)));
    MINF_WAIT_VMCNT(0);
    f32x16 sa[1][2], sb[1][2];
    qk_first(sa, buf.k(0));
    fresh(sa, d0);
    // iteration t: d0 = step t (logits in hand), d1 = step t+1 (K landed), d2 = step t+2
    int t = 0;
    while (h0) {
      iter(t, sa, sb);
      if (!h0) break;
      iter(t + 1, sb, sa);
      t += 2;
    }
    MINF_WAIT_VMCNT(0);      // the repeated loads of the last iterations
  }
};

// Three steps in flight per iteration, for contiguous steps: the matrix cores
// alternate between the logits of step t+1 (K Q^T) and the output update of
// step t-1 (V^T P^T) while the vector ALU turns the logits of step t into P(t).
// Every round then has the same mix -- 2 + 2 MFMAs, 2 logit pairs, 3 LDS reads,
// 2 tile loads -- which the two-deep scheme above cannot offer (its first rounds
// are all softmax, its last all MFMA, and one wave per SIMD issues in order).
// Price: V of step t-1 is read while V of step t waits and V of step t+1 lands:
// three V slots.  Iteration t issues K of step t+2 (rounds 0..3, needed at the
// top of iteration t+1) and then V of step t+1 (rounds 4..7, needed in
// iteration t+2); the single wait at the top leaves the 8 V loads in flight.
// The body is one straight path: without a current step P = 0 (infinite
// reference), without a next step the MFMAs form logits nobody consumes and
// the loads repeat an earlier step into the free slots; the first iteration
// multiplies a zero P(-1) with V(0).
template <class Gen, bool ROWS256>
struct WavePipe3 {
  Gen &gen;
  WaveState &st;
  const QAcc &qa;
  bool &has_ref;
  const LaneOfs &lo;
  StepBuf buf;
  const char *kh, *vh;       // head bases (bytes)
  unsigned k_rb, v_rb;
  const DmaLane &dk, &dv;
  MaskP mp;
  float c_log2;
  int lane;
  Step d0, d1, d2;          // steps t (softmax), t+1 (logits), t+2 (K fetch)
  bool h0, h1, h2, hp;      // ... exist; hp: step t-1 exists (its P awaits the output update)

  __device__ inline const char *row0(const char *head, unsigned rb, const Step &d) const {
    const unsigned kb = (unsigned)__builtin_amdgcn_readfirstlane(d.kbase);
    return head + (uint64_t)kb * rb;
  }
  __device__ inline void fresh(f32x16 (&s)[1][2], const Step &d) {
    if (d.cls == 2 || !has_ref) {
      MaskP m = mp;
      m.lo = d.lo; m.hi = d.hi;
      if (d.cls == 2) window_mask<1>(s, d.kbase, m, lane);
      if (!has_ref) special_tile<1>(s, st, d.kbase, m, false, true, c_log2, lane);
    }
    has_ref = true;
  }
  __device__ inline void qk_first(f32x16 (&s)[1][2], const char *tK) const {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const bf16x8 a = lds_read_k(tK, lo.k[ks]);
      if (ks == 0) {
        mfma_qk_first(s[0][0], a, qa.q[0][0]);
        mfma_qk_first(s[0][1], a, qa.q[1][0]);
      } else {
        mfma_qk_acc(s[0][0], a, qa.q[0][ks]);
        mfma_qk_acc(s[0][1], a, qa.q[1][ks]);
      }
    }
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 7" ::: "memory");   // results readable by the vector ALU
  }
  template <bool IS_K>
  __device__ inline void fetch_whole(const Step &d, unsigned dst) const {
    const char *a = row0(IS_K ? kh : vh, IS_K ? k_rb : v_rb, d);
    const unsigned rb = IS_K ? k_rb : v_rb;
    const unsigned (&vo)[4] = IS_K ? dk.voff : dv.voff;
    dma_pair<ROWS256, 0>(a, rb, vo, dst); dma_pair<ROWS256, 2>(a, rb, vo, dst);
    dma_pair<ROWS256, 4>(a, rb, vo, dst); dma_pair<ROWS256, 6>(a, rb, vo, dst);
  }

  // Iteration t with PH = t mod 6: K of step s lives in K slot s mod 2, V of step s in V slot
  // (s + 1) mod 3, so with the phase a template parameter every LDS address of the iteration is a
  // lane constant plus an immediate (the loop is unrolled six times; with the V slot in a register
  // every V operand read cost an address add on the vector ALU).
  static constexpr unsigned v_slot(int i) { return (unsigned)(2 + i) * HALF_BYTES; }
  template <int PH, bool FIRST>
  __device__ inline void iter(f32x16 (&s_cur)[1][2], f32x16 (&s_nxt)[1][2], bf16x8 (&p_prev)[2][2],
                              bf16x8 (&p_cur)[2][2]) {
    MINF_WAIT_VMCNT(8);      // K of step t+1 (and everything older) has landed; V of step t may be in flight
    const char *tK = buf.k((PH + 1) & 1);
    // V(t-1); in the very first iteration there is no step -1: zero P times the rows of V(0)
    const char *tV = buf.lds + v_slot(FIRST ? 1 : PH % 3);
    const unsigned k_dst = lds_addr_of(buf.k(PH & 1)), v_dst = lds_addr_of(buf.lds) + v_slot((PH + 2) % 3);
    const char *kt = row0(kh, k_rb, d2), *vt = row0(vh, v_rb, d1);
    bf16x8 kf[8], vf[8];
    kf[0] = lds_read_k(tK, lo.k[0]);
    auto fetch_v = [&](int i) {            // output update step i = (t, db)
      const int base = 16 * (i >> 2) * ROW_BYTES, db = i & 3;
      return lds_read_vt(tV, lo.v[db][0] + base, lo.v[db][1] + base);
    };
    vf[0] = fetch_v(0);
    const bool attend = h0;
    // no current step: infinite reference, P = exp2(-inf) = 0
    const float m0 = attend ? st.m[0] : INFINITY, m1 = attend ? st.m[1] : INFINITY;
    float lsum0 = 0.f, lsum1 = 0.f;
    // Pair e of the 16 logit pairs per lane, walked [t][nb][r]: round r handles pairs 2r, 2r + 1,
    // so that P(t) group (nb, tt) is born in the rounds in which P(t-1) group (., tt) is last used
    // and the two generations of P share registers.  The exponentials of pair e are issued first,
    // the sum and the conversion of pair e - 1 behind them (no wait state after a transcendental).
    float pe0 = 0.f, pe1 = 0.f;
    auto finish_pair = [&](int e) {        // pair e's exponentials are in pe0, pe1
      const int tt = e >> 3, nb = (e >> 2) & 1;
      if (nb == 0) lsum0 += pe0 + pe1; else lsum1 += pe0 + pe1;
      const f32x2 two = {pe0, pe1};
      unsigned pk = __builtin_bit_cast(unsigned, __builtin_convertvector(two, bf16x2));
      asm volatile("" : "+v"(pk), "+v"(lsum0), "+v"(lsum1));
      const bf16x2 b2 = __builtin_bit_cast(bf16x2, pk);
      p_cur[nb][tt][2 * (e & 3)] = b2[0];
      p_cur[nb][tt][2 * (e & 3) + 1] = b2[1];
    };
    // the two halves of a pair's work: exponentials of pair e; sum and conversion of the pair before
    float ne0 = 0.f, ne1 = 0.f;
    auto exp_pair = [&](int e) {
      const int tt = e >> 3, nb = (e >> 2) & 1, r = 8 * tt + 2 * (e & 3);
      const float m_use = nb == 0 ? m0 : m1;
      ne0 = fast_exp2(fmaf(s_cur[0][nb][r], c_log2, -m_use));
      ne1 = fast_exp2(fmaf(s_cur[0][nb][r + 1], c_log2, -m_use));
      asm volatile("" : "+v"(ne0), "+v"(ne1));
    };
    auto sum_pair = [&](int e) {           // finishes pair e - 1, then pair e's exponentials take its place
      if (e > 0) finish_pair(e - 1);
      pe0 = ne0; pe1 = ne1;
    };
    // One round = 4 groups, each opened by ONE MFMA and filled with about a quarter of the round's
    // other instructions: the wave issues in order, and a second MFMA right behind the first would
    // stall the issue for the 32 cycles the first occupies the pipeline -- time that is lost when
    // the round is bound by instruction issue, as it is here.
    auto round = [&](auto rc_) {
      constexpr int r = decltype(rc_)::value;
      // group 0: logits, query block 0; exponentials of pair 2r
      if (r == 0) mfma_qk_first(s_nxt[0][0], kf[0], qa.q[0][0]);
      else mfma_qk_acc(s_nxt[0][0], kf[r], qa.q[0][r]);
      exp_pair(2 * r);
      if (r + 1 < 8) kf[(r + 1) & 7] = lds_read_k(tK, lo.k[(r + 1) & 7]);
      __builtin_amdgcn_sched_barrier(0);
      // group 1: logits, query block 1; sum / conversion of pair 2r - 1; the round's two tile loads
      if (r == 0) mfma_qk_first(s_nxt[0][1], kf[0], qa.q[1][0]);
      else mfma_qk_acc(s_nxt[0][1], kf[r], qa.q[1][r]);
      sum_pair(2 * r);
      if (r < 4) dma_pair<ROWS256, 2 * (r & 3)>(kt, k_rb, dk.voff, k_dst);
      else dma_pair<ROWS256, 2 * (r & 3)>(vt, v_rb, dv.voff, v_dst);
      __builtin_amdgcn_sched_barrier(0);
      // group 2: output update step r, query block 0; exponentials of pair 2r + 1
      {
        const int tt = r >> 2, db = r & 3;
        st.o[db][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[r], p_prev[0][tt], st.o[db][0], 0, 0, 0);
      }
      exp_pair(2 * r + 1);
      if (r + 1 < 8) vf[(r + 1) & 7] = fetch_v((r + 1) & 7);
      __builtin_amdgcn_sched_barrier(0);
      // group 3: output update step r, query block 1; sum / conversion of pair 2r; bookkeeping
      {
        const int tt = r >> 2, db = r & 3;
        st.o[db][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[r], p_prev[1][tt], st.o[db][1], 0, 0, 0);
      }
      sum_pair(2 * r + 1);
      if (r == 7) finish_pair(15);
      if (r == 3) {
        // advance the generator between MFMAs
        hp = h0;
        d0 = d1; d1 = d2;
        h0 = h1; h1 = h2;
        Step dn = d2;
        h2 = h2 && gen.next(dn);
        if (h2) d2 = dn;
      }
      __builtin_amdgcn_sched_barrier(0);
    };
    round(std::integral_constant<int, 0>{});
    round(std::integral_constant<int, 1>{});
    round(std::integral_constant<int, 2>{});
    round(std::integral_constant<int, 3>{});
    round(std::integral_constant<int, 4>{});
    round(std::integral_constant<int, 5>{});
    round(std::integral_constant<int, 6>{});
    round(std::integral_constant<int, 7>{});
    if (attend) {
      st.l[0] += lsum0;
      st.l[1] += lsum1;
    }
    // after the generator advanced in round 3: d0 = the step whose logits are now in s_nxt
    if (h0) fresh(s_nxt, d0);
  }
  __device__ inline void run() {
    h0 = gen.next(d0);
    if (!h0) return;
    d1 = d0;
    h1 = gen.next(d1);
    d2 = d1;
    h2 = h1 && gen.next(d2);
    hp = false;
    // K of steps 0, 1 into K slots 0, 1; V of step 0 into V slot 1
    fetch_whole<true>(d0, lds_addr_of(buf.k(0)));
    fetch_whole<true>(d1, lds_addr_of(buf.k(1)));
    fetch_whole<false>(d0, lds_addr_of(buf.lds) + v_slot(1));
    MINF_WAIT_VMCNT(0);
    f32x16 sa[1][2], sb[1][2];
    bf16x8 pa[2][2], pb[2][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) (&pa[0][0])[i][j] = (__bf16)0.f;
    qk_first(sa, buf.k(0));
    fresh(sa, d0);
    // iteration t: d0 = step t (logits in hand), d1 = step t+1 (K landed), d2 = step t+2;
    // one iteration past the last step finishes its output update
    iter<0, true>(sa, sb, pa, pb);
    while (h0 || hp) {
      iter<1, false>(sb, sa, pb, pa);
      if (!(h0 || hp)) break;
      iter<2, false>(sa, sb, pa, pb);
      if (!(h0 || hp)) break;
      iter<3, false>(sb, sa, pb, pa);
      if (!(h0 || hp)) break;
      iter<4, false>(sa, sb, pa, pb);
      if (!(h0 || hp)) break;
      iter<5, false>(sb, sa, pb, pa);
      if (!(h0 || hp)) break;
      iter<0, false>(sa, sb, pa, pb);
    }
    MINF_WAIT_VMCNT(0);      // the repeated loads of the last iterations
  }
};

// ---------------------------------------------------------------------------
// Block-Sparse: one wave per (head, query block); steps = halves of the listed
// key blocks.
// ---------------------------------------------------------------------------
struct BsCtx {
  const bf16_t *kh, *vh;
  int64_t k_st, v_st;
  int N, NB, cnt;
  const int32_t *list;
  StepBuf buf;
  float c_log2;
};

template <int PASS>
__device__ inline void bs_pass(const BsCtx &c, WaveState &st, const LaneOfs &lo, const MaskP &mp, int lane) {
  // entries outside [0, NB) are skipped
  auto next_valid = [&](int i) {
    while (i < c.cnt) {
      const int b = c.list[i];
      if (b >= 0 && b < c.NB) break;
      ++i;
    }
    return i;
  };
  bool has_ref = false;
  int i = next_valid(0), half = 0, s = 0;
  if (i < c.cnt) fetch_step<true>(c.buf, 0, c.kh, c.vh, c.k_st, c.v_st, c.list[i] * BK, nullptr, c.N, lane);
  while (i < c.cnt) {
    const int kbase = c.list[i] * BK + 32 * half;
    int i2 = i;
    const int half2 = half ^ 1;
    if (half == 1) i2 = next_valid(i + 1);
    if (i2 < c.cnt) {
      fetch_step<true>(c.buf, s ^ 1, c.kh, c.vh, c.k_st, c.v_st, c.list[i2] * BK + 32 * half2, nullptr, c.N, lane);
      MINF_WAIT_VMCNT(16);
    } else {
      MINF_WAIT_VMCNT(0);
    }
    contiguous_step<1, PASS>(st, has_ref, lo, c.buf.k(s), c.buf.v(s), kbase, mp, c.c_log2, lane);
    i = i2; half = half2; s ^= 1;
  }
}

// Generator of the Block-Sparse steps: both halves of every listed block that
// holds a key some row may attend (ids outside [0, NB) and blocks past the
// diagonal are dropped).
struct BsGen {
  int mine;             // lane i: entry i of the current chunk of the block list
  int n, NB;
  const MaskP &mp;
  int i, half;
  __device__ inline bool next(Step &d) {
    while (i < n) {
      const int b = __builtin_amdgcn_readlane(mine, i);
      if (b >= 0 && b < NB) {
        const int kbase = b * BK + 32 * half;
        const int cls = classify_step<32>(kbase, mp);
        if (half == 1) { ++i; half = 0; } else half = 1;
        if (cls != 0) {
          d.kbase = kbase; d.lo = mp.lo; d.hi = mp.hi; d.cls = cls; d.cols = nullptr;
          return true;
        }
      } else {
        ++i; half = 0;
      }
    }
    return false;
  }
};

// One work item = one wave: query block b (a position in the processing order, if there is one) of list slot `slot`.
template <bool ROWS256>
__device__ __forceinline__ void bs_item(const QKV &x, const HeadList &hl, const int32_t *blk_idx,
                                        const int32_t *blk_cnt, const int32_t *order, int topk, int slot, int b,
                                        char *lds) {
  const int NB = x.N / BQ;
  if (order) {
    // position in the processing order -> query block (a permutation: every block is taken once)
    b = __builtin_amdgcn_readfirstlane(order[(int64_t)slot * NB + b]);
    if (b < 0 || b >= NB) return;
  }
  const int head = __builtin_amdgcn_readfirstlane(hl.h[slot]);
  const int kvh = to_sgpr(head / x.group);
  const bf16_t *qh = x.q + head * x.q_sh;
  bf16_t *oh = x.o + head * x.o_sh;
  const int lane = threadIdx.x;
  const int q0 = b * BQ;

  WaveState st;
  wave_init(st, qh, x.q_st, q0, lane);
  LaneOfs lo;
  lane_offsets(lo, lane);
  MaskP mp;
  mp.q0 = q0; mp.lo = 0; mp.hi = x.N; mp.n_init = KEY_NONE; mp.n_local = 1;
  BsCtx c;
  c.kh = x.k + kvh * x.k_sh; c.vh = x.v + kvh * x.v_sh; c.k_st = x.k_st; c.v_st = x.v_st;
  c.N = x.N; c.NB = NB; c.buf = StepBuf{lds}; c.c_log2 = x.c_log2;
  // the block list of this query block is walked 64 ids at a time, one per lane
  const int32_t *glist = blk_idx + ((int64_t)slot * NB + b) * topk;
  c.cnt = min(max(blk_cnt[(int64_t)slot * NB + b], 0), topk);
  c.list = glist;

  QAcc qa;
  pin_q(qa, st);
  DmaLane dk, dv;
  dma_lane_init(dk, x.k_st, lane);
  dma_lane_init(dv, x.v_st, lane);
  const int total = c.cnt;
  bool has_ref = false;
  for (int r0 = 0; r0 < total; r0 += 64) {
    const int n = min(total - r0, 64);
    const int mine = lane < n ? glist[r0 + lane] : -1;
    BsGen gen{mine, n, NB, mp, 0, 0};
    WavePipe3<BsGen, ROWS256> pipe{gen, st, qa, has_ref, lo, c.buf, reinterpret_cast<const char *>(c.kh),
                                   reinterpret_cast<const char *>(c.vh), (unsigned)x.k_st * 2u,
                                   (unsigned)x.v_st * 2u, dk, dv, mp, c.c_log2, lane};
    pipe.run();
  }
  if (needs_exact(st)) {
    load_q(st, qh, x.q_st, q0, lane);   // the pipelined pass kept Q in accumulator registers only
    reset_for_max_pass(st);
    bs_pass<PASS_MAX>(c, st, lo, mp, lane);
    finish_max_pass(st, x.c_log2);
    bs_pass<PASS_FIX>(c, st, lo, mp, lane);
  }
  wave_finish(st, oh, x.o_st, q0, lds, lane);
}

template <bool ROWS256>
__global__ __launch_bounds__(64) void bs_kernel(QKV x, HeadList hl, const int32_t *blk_idx,
                                                const int32_t *blk_cnt, const int32_t *order, int topk,
                                                Sched sched) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  int slot, b;
  if (!decode_wg(sched, slot, b)) return;
  bs_item<ROWS256>(x, hl, blk_idx, blk_cnt, order, topk, slot, b, lds);
}

// ---------------------------------------------------------------------------
// Vertical-Slash: one wave per (head, query block).
//  phase A: the slash runs [t0, t1) of the head, mapped to keys q0 - t, walked
//           32 keys at a time from the run's first key;
//  phase B: kept verticals that are causal for the block and outside every
//           run, compacted (ballot + prefix count) into LDS and gathered 32 at
//           a time.
// ---------------------------------------------------------------------------
struct VsCtx {
  const bf16_t *kh, *vh;
  int64_t k_st, v_st;
  int N, q0, n_v, n_c;
  const int32_t *vlist;
  const int2 *runs;
  const uint32_t *bits;
  StepBuf buf;
  int *cols;
  float c_log2;
};

template <int PASS>
__device__ inline void vs_pass(const VsCtx &c, WaveState &st, const LaneOfs &lo, MaskP mp, int lane) {
  const int q0 = c.q0;
  bool has_ref = false;
  // ---- phase A: slash runs -------------------------------------------------
  int iv = 0, ks = 0, ke = 0, pos = 0;   // run index, clipped key range [ks, ke), next step start
  auto next_run_step = [&](int &kbase, int &rlo, int &rhi) -> bool {
    while (true) {
      if (pos < ke) {
        kbase = pos; rlo = ks; rhi = ke;
        pos += 32;
        return true;
      }
      if (iv >= c.n_c) return false;
      const int2 r = c.runs[iv];
      if (r.x > q0) { iv = c.n_c; return false; }   // runs ascend: no later run reaches key >= 0
      ++iv;
      ks = max(q0 - r.y + 1, 0);
      ke = min(q0 - r.x + 1, c.N);
      pos = ks;
    }
  };
  int s = 0;
  int kb, rlo, rhi, kb2 = 0, rlo2 = 0, rhi2 = 0;
  bool have = next_run_step(kb, rlo, rhi);
  if (have) fetch_step<true>(c.buf, 0, c.kh, c.vh, c.k_st, c.v_st, kb, nullptr, c.N, lane);
  while (have) {
    const bool have2 = next_run_step(kb2, rlo2, rhi2);
    if (have2) {
      fetch_step<true>(c.buf, s ^ 1, c.kh, c.vh, c.k_st, c.v_st, kb2, nullptr, c.N, lane);
      MINF_WAIT_VMCNT(16);
    } else {
      MINF_WAIT_VMCNT(0);
    }
    mp.lo = rlo; mp.hi = rhi;
    contiguous_step<1, PASS>(st, has_ref, lo, c.buf.k(s), c.buf.v(s), kb, mp, c.c_log2, lane);
    have = have2; kb = kb2; rlo = rlo2; rhi = rhi2; s ^= 1;
  }

  // ---- phase B: verticals ----------------------------------------------------
  const int qlast = q0 + BQ - 1;
  int *cols = c.cols;
  int vpos = 0;                       // next entry of vlist to examine
  while (vpos < c.n_v) {
    // compact up to VCAP columns into cols[]
    int ncol = 0;
    while (vpos < c.n_v && ncol <= VCAP - 64) {
      const int i = vpos + lane;
      const int v = i < c.n_v ? c.vlist[i] : KEY_NONE;
      bool ok = v <= qlast && v >= 0;
      if (ok) {
        const int t = q0 - v + 64;     // bit index of offset q0 - v, in [1, q0 + 64]
        ok = ((c.bits[t >> 5] >> (t & 31)) & 1u) == 0u;
      }
      const unsigned long long bal = __builtin_amdgcn_ballot_w64(ok);
      const int before = __builtin_popcountll(bal & ((1ull << lane) - 1ull));
      if (ok) cols[ncol + before] = v;
      ncol += __builtin_popcountll(bal);
      vpos += 64;
      // the list ascends: once a whole chunk is past the block nothing follows
      if (__shfl(v, 0) > qlast) { vpos = c.n_v; break; }
    }
    if (ncol == 0) continue;
    const int nstep = (ncol + 31) / 32;
    if (lane + ncol < nstep * 32) cols[ncol + lane] = KEY_NONE;   // pad the last step
    wave_lds_sync();                   // cols[] visible to every lane (earlier tile loads were awaited)
    fetch_step<false>(c.buf, s, c.kh, c.vh, c.k_st, c.v_st, 0, cols, c.N, lane);
    for (int t = 0; t < nstep; ++t) {
      if (t + 1 < nstep) {
        fetch_step<false>(c.buf, s ^ 1, c.kh, c.vh, c.k_st, c.v_st, 0, cols + (t + 1) * 32, c.N, lane);
        MINF_WAIT_VMCNT(16);
      } else {
        MINF_WAIT_VMCNT(0);
      }
      gathered_step<1, PASS>(st, has_ref, lo, c.buf.k(s), c.buf.v(s), cols + t * 32, mp, c.c_log2, lane);
      s ^= 1;
    }
    wave_lds_sync();                   // every lane is done with cols[] before the next round refills it
  }
}

// Generators of the Vertical-Slash steps for the pipelined pass.
// Slash runs: a chunk of 64 runs held one per lane, each walked 32 keys at a time.
struct VsRunGen {
  int2 mine;            // lane i: run i of the chunk
  int n, q0, N;
  int iv, ks, ke, pos;
  __device__ inline bool next(Step &d) {
    while (true) {
      if (pos < ke) {
        // the step covers the keys pos .. pos+31 of the run; near the end of the
        // sequence its 32 fetched rows are shifted back to stay inside [0, N) and
        // the window's lower bound hides the rows the step before already took
        d.kbase = min(pos, N - 32); d.lo = pos; d.hi = ke; d.cols = nullptr;
        // the run is causal up to q0 + 63 by construction; only the key window and
        // the diagonal can mask elements
        d.cls = (d.kbase == pos && pos + 31 < ke && pos + 31 <= q0) ? 1 : 2;
        pos += 32;
        return true;
      }
      if (iv >= n) return false;
      const int rx = __builtin_amdgcn_readlane(mine.x, iv), ry = __builtin_amdgcn_readlane(mine.y, iv);
      ++iv;
      ks = max(q0 - ry + 1, 0);
      ke = min(q0 - rx + 1, N);
      pos = ks;
    }
  }
};

// Gathered verticals: steps of 32 entries of the compacted column list (LDS).
struct VsColGen {
  const int *cols;
  int nstep, q0, t;
  __device__ inline bool next(Step &d) {
    if (t >= nstep) return false;
    d.kbase = 0; d.lo = 0; d.hi = 0;
    d.cols = cols + 32 * t;
    d.cls = d.cols[31] <= q0 ? 1 : 2;     // ascending list: the last entry decides (KEY_NONE pads)
    ++t;
    return true;
  }
};

// Phase B of the optimistic pass: the kept verticals that are causal for the block and outside
// every run, compacted into this wave's column list and gathered 32 per step through this wave's
// own ring.  No workgroup barrier: every wave has its own list length.
template <bool ROWS256>
__device__ inline void vs_cols_pipelined(const VsCtx &c, WaveState &st, const QAcc &qa, bool &has_ref,
                                         const LaneOfs &lo, const MaskP &mp, const DmaLane &dk,
                                         const DmaLane &dv, int lane) {
  const int q0 = c.q0;
  const char *khb = reinterpret_cast<const char *>(c.kh), *vhb = reinterpret_cast<const char *>(c.vh);
  const unsigned k_rb = (unsigned)c.k_st * 2u, v_rb = (unsigned)c.v_st * 2u;
  const int qlast = q0 + BQ - 1;
  int *cols = c.cols;
  int vpos = 0;
  while (vpos < c.n_v) {
    int ncol = 0;
    while (vpos < c.n_v && ncol <= VCAP - 64) {
      const int i = vpos + lane;
      const int v = i < c.n_v ? c.vlist[i] : KEY_NONE;
      bool ok = v <= qlast && v >= 0;
      if (ok) {
        const int t = q0 - v + 64;     // bit index of offset q0 - v, in [1, q0 + 64]
        ok = ((c.bits[t >> 5] >> (t & 31)) & 1u) == 0u;
      }
      const unsigned long long bal = __builtin_amdgcn_ballot_w64(ok);
      const int before = __builtin_popcountll(bal & ((1ull << lane) - 1ull));
      if (ok) cols[ncol + before] = v;
      ncol += __builtin_popcountll(bal);
      vpos += 64;
      if (__shfl(v, 0) > qlast) { vpos = c.n_v; break; }
    }
    if (ncol == 0) continue;
    const int nstep = (ncol + 31) / 32;
    if (lane + ncol < nstep * 32) cols[ncol + lane] = KEY_NONE;   // pad the last step
    wave_lds_sync();
    VsColGen gen{cols, nstep, q0, 0};
    WavePipe<VsColGen, true, ROWS256> pipe{gen, st, qa, has_ref, lo, c.buf, khb, vhb, k_rb, v_rb, dk, dv, c.N, mp, c.c_log2, lane};
    pipe.run();
    wave_lds_sync();
  }
}

// Optimistic pass of the Vertical-Slash kernel, software pipelined.
template <bool ROWS256>
__device__ inline void vs_pass_pipelined(const VsCtx &c, WaveState &st, const LaneOfs &lo, const MaskP &mp,
                                         int lane) {
  const int q0 = c.q0;
  bool has_ref = false;
  QAcc qa;
  pin_q(qa, st);
  DmaLane dk, dv;
  dma_lane_init(dk, c.k_st, lane);
  dma_lane_init(dv, c.v_st, lane);
  const char *khb = reinterpret_cast<const char *>(c.kh), *vhb = reinterpret_cast<const char *>(c.vh);
  const unsigned k_rb = (unsigned)c.k_st * 2u, v_rb = (unsigned)c.v_st * 2u;
  // ---- phase A: slash runs, 64 at a time, one per lane (the run list takes no LDS)
  for (int r0 = 0; r0 < c.n_c; r0 += 64) {
    const int n = min(c.n_c - r0, 64);
    int2 mine = make_int2(KEY_NONE, KEY_NONE);
    if (lane < n) mine = c.runs[r0 + lane];
    // runs ascend: those that reach a key >= 0 (t0 <= q0) form a prefix
    const int usable = __builtin_popcountll(__builtin_amdgcn_ballot_w64(lane < n && mine.x <= q0));
    if (usable == 0) break;
    VsRunGen gen{mine, usable, q0, c.N, 0, 0, 0, 0};
    WavePipe3<VsRunGen, ROWS256> pipe{gen, st, qa, has_ref, lo, c.buf, khb, vhb, k_rb, v_rb, dk, dv, mp, c.c_log2, lane};
    pipe.run();
    if (usable < n) break;
  }
  vs_cols_pipelined<ROWS256>(c, st, qa, has_ref, lo, mp, dk, dv, lane);
}

// One work item = one wave: query block b of list slot `slot`.
template <bool ROWS256>
__device__ __forceinline__ void vs_item(const QKV &x, const HeadList &hl, const int32_t *v_idx,
                                        const int32_t *cover, const uint32_t *cover_bits,
                                        const int32_t *counts, int nv, int ns, int cover_words, int slot, int b,
                                        char *lds) {
  const int head = __builtin_amdgcn_readfirstlane(hl.h[slot]);
  const int kvh = to_sgpr(head / x.group);
  const bf16_t *qh = x.q + head * x.q_sh;
  bf16_t *oh = x.o + head * x.o_sh;
  const int lane = threadIdx.x;
  const int q0 = b * BQ;

  VsCtx c;
  c.kh = x.k + kvh * x.k_sh; c.vh = x.v + kvh * x.v_sh; c.k_st = x.k_st; c.v_st = x.v_st;
  // The column list of the vertical phase, which runs two deep on V slots 0 and 1, lives in V slot 2.
  c.N = x.N; c.q0 = q0; c.buf = StepBuf{lds}; c.c_log2 = x.c_log2;
  c.cols = reinterpret_cast<int *>(lds + 4 * HALF_BYTES);   // [VCAP + 64]
  c.n_v = min(max(counts[slot * 4 + 0], 0), nv);
  c.n_c = min(max(counts[slot * 4 + 2], 0), ns);
  c.vlist = v_idx + (int64_t)slot * nv;
  c.runs = reinterpret_cast<const int2 *>(cover) + (int64_t)slot * ns;
  c.bits = cover_bits + (int64_t)slot * cover_words;

  WaveState st;
  wave_init(st, qh, x.q_st, q0, lane);
  LaneOfs lo;
  lane_offsets(lo, lane);
  MaskP mp;
  mp.q0 = q0; mp.n_init = KEY_NONE; mp.n_local = 1; mp.lo = 0; mp.hi = 0;

  vs_pass_pipelined<ROWS256>(c, st, lo, mp, lane);
  if (needs_exact(st)) {
    load_q(st, qh, x.q_st, q0, lane);   // the pipelined pass kept Q in accumulator registers only
    reset_for_max_pass(st);
    vs_pass<PASS_MAX>(c, st, lo, mp, lane);
    finish_max_pass(st, x.c_log2);
    vs_pass<PASS_FIX>(c, st, lo, mp, lane);
  }
  wave_finish(st, oh, x.o_st, q0, lds, lane);
}

template <bool ROWS256>
__global__ __launch_bounds__(64) void vs_kernel(QKV x, HeadList hl, const int32_t *v_idx,
                                                const int32_t *cover, const uint32_t *cover_bits,
                                                const int32_t *counts, int nv, int ns, int cover_words,
                                                Sched sched) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  int slot, b;
  if (!decode_wg(sched, slot, b)) return;
  vs_item<ROWS256>(x, hl, v_idx, cover, cover_bits, counts, nv, ns, cover_words, slot, b, lds);
}

// Vertical-Slash and Block-Sparse heads of a layer in ONE launch (the layers of the paper's models
// mix the patterns, App. E): the work items of the two kinds are interleaved four to one in
// launch order, each kind keeping its own XCD-aware mapping (a workgroup id's low three bits are
// the XCD in both), so that every XCD holds both kinds at any time.  Same results as the two
// separate launches, bit for bit; measured slower than them (the Block-Sparse items stream other
// K/V heads through the L2s that the Vertical-Slash items share) and therefore not what
// minf_vs_attn / minf_bs_attn do: kept as the measured alternative.
struct VsArgs {
  const int32_t *v_idx, *cover;
  const uint32_t *cover_bits;
  const int32_t *counts;
  int nv, ns, cover_words;
};
struct BsArgs {
  const int32_t *blk_idx, *blk_cnt, *order;
  int topk;
};
template <bool ROWS256>
__global__ __launch_bounds__(64) void vs_bs_kernel(QKV x, HeadList hv, VsArgs va, Sched sv, HeadList hb, BsArgs ba,
                                                   Sched sb) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  int kind, slot, b;
  if (!decode_mixed(sv, sb, blockIdx.x, kind, slot, b)) return;
  if (kind == 0)
    vs_item<ROWS256>(x, hv, va.v_idx, va.cover, va.cover_bits, va.counts, va.nv, va.ns, va.cover_words, slot, b, lds);
  else
    bs_item<ROWS256>(x, hb, ba.blk_idx, ba.blk_cnt, ba.order, ba.topk, slot, b, lds);
}

// ---------------------------------------------------------------------------
// Vertical-Slash, shared tiles: a workgroup is four waves = four consecutive
// query blocks of one head.  The key sequence of a slash run is the same for
// every query block up to a shift by the block's first row (App. C.4.2: the
// slash tiles are translation invariant), so the four waves walk one common
// schedule of 32-key steps, each wave two steps behind the one before it; waves
// that are inside the same run then need the same 32 keys at the same moment
// and only the first of them (the "leader") fetches them, into its own ring
// (see vs_ring_sched.h).  Every wave still computes only its own tiles.
// LDS: four rings of 2 K + 3 V slots of 8 KiB (160 KiB); ring slots are
// indexed by the step number, which is common to the four waves.
// ---------------------------------------------------------------------------
constexpr int RING_BYTES = 5 * HALF_BYTES;

// The runs of a head, 64 at a time one per lane; the next 64 are fetched when the schedule
// reaches them (once per 64 runs; the load waits for the tile loads in flight).
struct RunLanes {
  const int2 *runs;
  int n_c, lane, base;
  int2 mine;
  __device__ inline void load(int b) {
    base = b;
    mine = make_int2(KEY_NONE, KEY_NONE);
    if (b + lane < n_c) mine = runs[b + lane];
  }
  __device__ inline bool operator()(int iv, int &a, int &b) {
    if (iv >= n_c) return false;
    if (iv - base >= 64) load(base + 64);
    a = __builtin_amdgcn_readlane(mine.x, iv - base);
    b = __builtin_amdgcn_readlane(mine.y, iv - base);
    return true;
  }
};

// The three-stream pipeline of WavePipe3 for four waves in lock step.  Differences:
//  - the rows of a step live in the ring of the step's leader (RStep::src); a wave issues the
//    tile loads of a step only if it is that leader (RStep::load);
//  - one workgroup barrier at the top of every iteration, behind the wait for the wave's own
//    loads: the leader's rows are then visible to its followers, and every wave is done reading
//    the slots this iteration's loads overwrite;
//  - a step with nothing to attend (the idle steps of the skew, steps of a run that lie
//    before key 0 for this wave only) is run with P = 0.  The rings are zero-filled at the start
//    and only ever receive K/V rows, so what such a step multiplies by zero is finite.
template <class Gen, bool ROWS256>
struct RingPipe3 {
  Gen &gen;
  WaveState &st;
  const QAcc &qa;
  bool &has_ref;
  const LaneOfs &lo;
  char *lds0;                // ring of wave w at lds0 + w * RING_BYTES
  int wave;
  const char *kh, *vh;       // head bases (bytes)
  unsigned k_rb, v_rb;
  const DmaLane &dk, &dv;
  MaskP mp;
  float c_log2;
  int lane;
  RStep d0, d1, d2;          // steps t (softmax), t+1 (logits), t+2 (K fetch)
  bool h0, h1, h2, hp;       // ... exist; hp: step t-1 exists (its P awaits the output update)
  int src_p;                 // ring that holds V of step t-1

  static constexpr unsigned k_slot(int i) { return (unsigned)i * HALF_BYTES; }
  static constexpr unsigned v_slot(int i) { return (unsigned)(2 + i) * HALF_BYTES; }
  __device__ inline char *ring(int w) const { return lds0 + w * RING_BYTES; }
  __device__ inline const char *row0(const char *head, unsigned rb, const RStep &d) const {
    const unsigned kb = (unsigned)__builtin_amdgcn_readfirstlane(d.kbase);
    return head + (uint64_t)kb * rb;
  }
  __device__ inline void barrier() const { asm volatile("s_barrier" ::: "memory"); }
  // element mask and / or exponent reference on the fresh logits of a step (nothing for a step
  // without work: its logits are never used)
  __device__ inline void fresh(f32x16 (&s)[1][2], const RStep &d) {
    if (d.mask || (d.work && !has_ref)) {
      MaskP m = mp;
      m.lo = d.lo; m.hi = d.hi;
      if (d.mask) window_mask<1>(s, d.kbase, m, lane);
      if (!has_ref) special_tile<1>(s, st, d.kbase, m, false, true, c_log2, lane);
    }
    has_ref = has_ref || d.work;
  }
  __device__ inline void qk_first(f32x16 (&s)[1][2], const char *tK) const {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const bf16x8 a = lds_read_k(tK, lo.k[ks]);
      if (ks == 0) {
        mfma_qk_first(s[0][0], a, qa.q[0][0]);
        mfma_qk_first(s[0][1], a, qa.q[1][0]);
      } else {
        mfma_qk_acc(s[0][0], a, qa.q[0][ks]);
        mfma_qk_acc(s[0][1], a, qa.q[1][ks]);
      }
    }
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 7" ::: "memory");   // results readable by the vector ALU
  }
  template <bool IS_K>
  __device__ inline void fetch_whole(const RStep &d, unsigned dst) const {
    const char *a = row0(IS_K ? kh : vh, IS_K ? k_rb : v_rb, d);
    const unsigned rb = IS_K ? k_rb : v_rb;
    const unsigned (&vo)[4] = IS_K ? dk.voff : dv.voff;
    dma_pair<ROWS256, 0>(a, rb, vo, dst); dma_pair<ROWS256, 2>(a, rb, vo, dst);
    dma_pair<ROWS256, 4>(a, rb, vo, dst); dma_pair<ROWS256, 6>(a, rb, vo, dst);
  }

  // Iteration t with PH = t mod 6: K of step s lives in K slot s mod 2, V of step s in V slot
  // (s + 1) mod 3 of the leader's ring.
  template <int PH, bool FIRST>
  __device__ inline void iter(f32x16 (&s_cur)[1][2], f32x16 (&s_nxt)[1][2], bf16x8 (&p_prev)[2][2],
                              bf16x8 (&p_cur)[2][2]) {
    // Outstanding loads of this wave: K of step t+1, then V of step t (eight each, if this wave
    // leads those steps).  K must have landed, and so must V of step t-1 (older than both).
    if (h0 && d0.load) MINF_WAIT_VMCNT(8); else MINF_WAIT_VMCNT(0);
    barrier();
    const char *tK = ring(d1.src) + k_slot((PH + 1) & 1);
    // V(t-1); in the very first iteration there is no step -1: zero P times the rows of V(0)
    const char *tV = ring(FIRST ? d0.src : src_p) + v_slot(FIRST ? 1 : PH % 3);
    const unsigned k_dst = lds_addr_of(ring(wave)) + k_slot(PH & 1);
    const unsigned v_dst = lds_addr_of(ring(wave)) + v_slot((PH + 2) % 3);
    const bool ld_k = h2 && d2.load, ld_v = h1 && d1.load;
    const char *kt = row0(kh, k_rb, d2), *vt = row0(vh, v_rb, d1);
    bf16x8 kf[8], vf[8];
    kf[0] = lds_read_k(tK, lo.k[0]);
    auto fetch_v = [&](int i) {            // output update step i = (t, db)
      const int base = 16 * (i >> 2) * ROW_BYTES, db = i & 3;
      return lds_read_vt(tV, lo.v[db][0] + base, lo.v[db][1] + base);
    };
    vf[0] = fetch_v(0);
    const bool attend = h0 && d0.work;
    // nothing to attend: infinite reference, P = exp2(-inf) = 0
    const float m0 = attend ? st.m[0] : INFINITY, m1 = attend ? st.m[1] : INFINITY;
    float lsum0 = 0.f, lsum1 = 0.f;
    float pe0 = 0.f, pe1 = 0.f;
    auto finish_pair = [&](int e) {        // pair e's exponentials are in pe0, pe1
      const int tt = e >> 3, nb = (e >> 2) & 1;
      if (nb == 0) lsum0 += pe0 + pe1; else lsum1 += pe0 + pe1;
      const f32x2 two = {pe0, pe1};
      unsigned pk = __builtin_bit_cast(unsigned, __builtin_convertvector(two, bf16x2));
      asm volatile("" : "+v"(pk), "+v"(lsum0), "+v"(lsum1));
      const bf16x2 b2 = __builtin_bit_cast(bf16x2, pk);
      p_cur[nb][tt][2 * (e & 3)] = b2[0];
      p_cur[nb][tt][2 * (e & 3) + 1] = b2[1];
    };
    float ne0 = 0.f, ne1 = 0.f;
    auto exp_pair = [&](int e) {
      const int tt = e >> 3, nb = (e >> 2) & 1, r = 8 * tt + 2 * (e & 3);
      const float m_use = nb == 0 ? m0 : m1;
      ne0 = fast_exp2(fmaf(s_cur[0][nb][r], c_log2, -m_use));
      ne1 = fast_exp2(fmaf(s_cur[0][nb][r + 1], c_log2, -m_use));
      asm volatile("" : "+v"(ne0), "+v"(ne1));
    };
    auto sum_pair = [&](int e) {           // finishes pair e - 1, then pair e's exponentials take its place
      if (e > 0) finish_pair(e - 1);
      pe0 = ne0; pe1 = ne1;
    };
    // the round structure is that of WavePipe3: four groups, each opened by one MFMA
    auto round = [&](auto rc_) {
      constexpr int r = decltype(rc_)::value;
      if (r == 0) mfma_qk_first(s_nxt[0][0], kf[0], qa.q[0][0]);
      else mfma_qk_acc(s_nxt[0][0], kf[r], qa.q[0][r]);
      exp_pair(2 * r);
      if (r + 1 < 8) kf[(r + 1) & 7] = lds_read_k(tK, lo.k[(r + 1) & 7]);
      __builtin_amdgcn_sched_barrier(0);
      if (r == 0) mfma_qk_first(s_nxt[0][1], kf[0], qa.q[1][0]);
      else mfma_qk_acc(s_nxt[0][1], kf[r], qa.q[1][r]);
      sum_pair(2 * r);
      if (r < 4) {
        if (ld_k) dma_pair<ROWS256, 2 * (r & 3)>(kt, k_rb, dk.voff, k_dst);
      } else {
        if (ld_v) dma_pair<ROWS256, 2 * (r & 3)>(vt, v_rb, dv.voff, v_dst);
      }
      __builtin_amdgcn_sched_barrier(0);
      {
        const int tt = r >> 2, db = r & 3;
        st.o[db][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[r], p_prev[0][tt], st.o[db][0], 0, 0, 0);
      }
      exp_pair(2 * r + 1);
      if (r + 1 < 8) vf[(r + 1) & 7] = fetch_v((r + 1) & 7);
      __builtin_amdgcn_sched_barrier(0);
      {
        const int tt = r >> 2, db = r & 3;
        st.o[db][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[r], p_prev[1][tt], st.o[db][1], 0, 0, 0);
      }
      sum_pair(2 * r + 1);
      if (r == 7) finish_pair(15);
      if (r == 3) {
        // advance the generator between MFMAs
        hp = h0;
        src_p = d0.src;
        d0 = d1; d1 = d2;
        h0 = h1; h1 = h2;
        RStep dn = d2;
        h2 = h2 && gen.next(dn);
        if (h2) d2 = dn;
      }
      __builtin_amdgcn_sched_barrier(0);
    };
    round(std::integral_constant<int, 0>{});
    round(std::integral_constant<int, 1>{});
    round(std::integral_constant<int, 2>{});
    round(std::integral_constant<int, 3>{});
    round(std::integral_constant<int, 4>{});
    round(std::integral_constant<int, 5>{});
    round(std::integral_constant<int, 6>{});
    round(std::integral_constant<int, 7>{});
    if (attend) {
      st.l[0] += lsum0;
      st.l[1] += lsum1;
    }
    // after the generator advanced in round 3: d0 = the step whose logits are now in s_nxt
    if (h0) fresh(s_nxt, d0);
  }
  // Every wave of the workgroup must call this, and the generators of the four waves must yield
  // the same number of steps: the iterations meet at barriers.
  __device__ inline void run() {
    h0 = gen.next(d0);
    if (!h0) return;
    d1 = d0;
    h1 = gen.next(d1);
    d2 = d1;
    h2 = h1 && gen.next(d2);
    hp = false;
    src_p = wave;
    // K of steps 0, 1 into K slots 0, 1; V of step 0 into V slot 1 (leaders only)
    if (d0.load) fetch_whole<true>(d0, lds_addr_of(ring(wave)) + k_slot(0));
    if (h1 && d1.load) fetch_whole<true>(d1, lds_addr_of(ring(wave)) + k_slot(1));
    if (d0.load) fetch_whole<false>(d0, lds_addr_of(ring(wave)) + v_slot(1));
    MINF_WAIT_VMCNT(0);
    barrier();
    f32x16 sa[1][2], sb[1][2];
    bf16x8 pa[2][2], pb[2][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) (&pa[0][0])[i][j] = (__bf16)0.f;
    qk_first(sa, ring(d0.src) + k_slot(0));
    fresh(sa, d0);
    iter<0, true>(sa, sb, pa, pb);
    while (h0 || hp) {
      iter<1, false>(sb, sa, pb, pa);
      if (!(h0 || hp)) break;
      iter<2, false>(sa, sb, pa, pb);
      if (!(h0 || hp)) break;
      iter<3, false>(sb, sa, pb, pa);
      if (!(h0 || hp)) break;
      iter<4, false>(sa, sb, pa, pb);
      if (!(h0 || hp)) break;
      iter<5, false>(sb, sa, pb, pa);
      if (!(h0 || hp)) break;
      iter<0, false>(sa, sb, pa, pb);
    }
    MINF_WAIT_VMCNT(0);
    barrier();               // the followers are done with this wave's ring
  }
};

template <bool ROWS256>
__global__ __launch_bounds__(256) void vs_ring_kernel(QKV x, HeadList hl, const int32_t *v_idx,
                                                      const int32_t *cover, const uint32_t *cover_bits,
                                                      const int32_t *counts, int nv, int ns, int cover_words,
                                                      Sched sched) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int NB = x.N / BQ;
  int slot, sb;
  if (!decode_wg(sched, slot, sb)) return;
  const int head = __builtin_amdgcn_readfirstlane(hl.h[slot]);
  const int kvh = to_sgpr(head / x.group);
  const bf16_t *qh = x.q + head * x.q_sh;
  bf16_t *oh = x.o + head * x.o_sh;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int blk = sb * 4 + wave;
  // A wave past the last block runs the common schedule on the rows of the last block (the
  // barriers need it) with the masks of its virtual position; it writes nothing.
  const bool active = blk < NB;
  const int q0 = blk * BQ;
  char *ring = lds + wave * RING_BYTES;

  // rings start as zeros: a step that attends nothing multiplies their content by P = 0
#pragma unroll
  for (int i = 0; i < RING_BYTES / (64 * 16); ++i)
    *reinterpret_cast<uint4 *>(ring + (i * 64 + lane) * 16) = make_uint4(0u, 0u, 0u, 0u);

  VsCtx c;
  c.kh = x.k + kvh * x.k_sh; c.vh = x.v + kvh * x.v_sh; c.k_st = x.k_st; c.v_st = x.v_st;
  c.N = x.N; c.q0 = q0; c.buf = StepBuf{ring}; c.c_log2 = x.c_log2;
  c.cols = reinterpret_cast<int *>(ring + 4 * HALF_BYTES);   // [VCAP + 64], third V slot
  c.n_v = min(max(counts[slot * 4 + 0], 0), nv);
  c.n_c = min(max(counts[slot * 4 + 2], 0), ns);
  c.vlist = v_idx + (int64_t)slot * nv;
  c.runs = reinterpret_cast<const int2 *>(cover) + (int64_t)slot * ns;
  c.bits = cover_bits + (int64_t)slot * cover_words;

  WaveState st;
  wave_init(st, qh, x.q_st, active ? q0 : (NB - 1) * BQ, lane);
  LaneOfs lo;
  lane_offsets(lo, lane);
  MaskP mp;
  mp.q0 = q0; mp.n_init = KEY_NONE; mp.n_local = 1; mp.lo = 0; mp.hi = 0;
  __syncthreads();

  bool has_ref = false;
  QAcc qa;
  pin_q(qa, st);
  DmaLane dk, dv;
  dma_lane_init(dk, c.k_st, lane);
  dma_lane_init(dv, c.v_st, lane);
  {
    // ---- phase A: slash runs, shared between the four waves
    RunLanes rl{c.runs, c.n_c, lane, 0, make_int2(KEY_NONE, KEY_NONE)};
    rl.load(0);
    VsRingGen<RunLanes> gen(rl, sb * 4 * BQ, wave, c.N);
    RingPipe3<VsRingGen<RunLanes>, ROWS256> pipe{gen, st, qa, has_ref, lo, lds, wave,
                                                 reinterpret_cast<const char *>(c.kh),
                                                 reinterpret_cast<const char *>(c.vh), (unsigned)c.k_st * 2u,
                                                 (unsigned)c.v_st * 2u, dk, dv, mp, c.c_log2, lane};
    pipe.run();
  }
  if (!active) return;       // no workgroup barrier below this line
  // ---- phase B: verticals, per wave
  vs_cols_pipelined<ROWS256>(c, st, qa, has_ref, lo, mp, dk, dv, lane);
  if (needs_exact(st)) {
    load_q(st, qh, x.q_st, q0, lane);   // the pipelined pass kept Q in accumulator registers only
    reset_for_max_pass(st);
    vs_pass<PASS_MAX>(c, st, lo, mp, lane);
    finish_max_pass(st, x.c_log2);
    vs_pass<PASS_FIX>(c, st, lo, mp, lane);
  }
  wave_finish(st, oh, x.o_st, q0, ring, lane);
}

// ---------------------------------------------------------------------------
// host-side launches
// ---------------------------------------------------------------------------
static hipError_t set_lds(const void *fn, size_t bytes) {
  return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

hipError_t launch_ashape(const QKV &x, const HeadList &hl, int n_init, int n_local, hipStream_t st) {
  const int NB = x.N / BQ, NSB = (NB + 3) / 4;
  const Sched s = make_sched(hl, x.group, NSB);
  const size_t lds = 8 * TILE_BYTES;   // four K and four V slots
  // rows 256 bytes apart in both K and V (the [head][token][128] layout): cheaper tile fetch
  const bool rows256 = x.k_st == D && x.v_st == D;
  const void *fn = rows256 ? reinterpret_cast<const void *>(ashape_kernel<true>)
                           : reinterpret_cast<const void *>(ashape_kernel<false>);
  hipError_t e = set_lds(fn, lds);
  if (e != hipSuccess) return e;
  if (rows256)
    hipLaunchKernelGGL(ashape_kernel<true>, dim3(s.per_xcd * 8), dim3(256), lds, st, x, hl, n_init, n_local, s);
  else
    hipLaunchKernelGGL(ashape_kernel<false>, dim3(s.per_xcd * 8), dim3(256), lds, st, x, hl, n_init, n_local, s);
  return hipGetLastError();
}

hipError_t launch_bs(const QKV &x, const HeadList &hl, const int32_t *blk_idx, const int32_t *blk_cnt,
                     const int32_t *order, int topk, hipStream_t st) {
  const int NB = x.N / BQ;
  const Sched s = make_sched(hl, x.group, NB);
  const size_t lds = 5 * HALF_BYTES;
  const bool rows256 = x.k_st == D && x.v_st == D;
  const void *fn = rows256 ? reinterpret_cast<const void *>(bs_kernel<true>)
                           : reinterpret_cast<const void *>(bs_kernel<false>);
  hipError_t e = set_lds(fn, lds);
  if (e != hipSuccess) return e;
  if (rows256)
    hipLaunchKernelGGL(bs_kernel<true>, dim3(s.per_xcd * 8), dim3(64), lds, st, x, hl, blk_idx, blk_cnt, order, topk, s);
  else
    hipLaunchKernelGGL(bs_kernel<false>, dim3(s.per_xcd * 8), dim3(64), lds, st, x, hl, blk_idx, blk_cnt, order, topk, s);
  return hipGetLastError();
}

hipError_t launch_vs(const QKV &x, const HeadList &hl, const int32_t *v_idx, const int32_t *cover,
                     const uint32_t *cover_bits, const int32_t *counts, int nv, int ns,
                     int cover_words, hipStream_t st) {
  const int NB = x.N / BQ;
  // gathered rows are addressed with 32-bit byte offsets from the head base (checked by the caller)
  const bool rows256 = x.k_st == D && x.v_st == D;
  // MINF_VS_ENGINE=ring selects the shared-tile engine (four waves per workgroup, slash-run tiles
  // fetched once per group of waves); it is slower than the default on every measured workload
  // and kept as a measured alternative.
  const bool use_ring = getenv("MINF_VS_ENGINE") != nullptr && strcmp(getenv("MINF_VS_ENGINE"), "ring") == 0;
  if (use_ring) {
    const Sched s = make_sched(hl, x.group, (NB + 3) / 4);
    const size_t lds = 4 * RING_BYTES;
    const void *fn = rows256 ? reinterpret_cast<const void *>(vs_ring_kernel<true>)
                             : reinterpret_cast<const void *>(vs_ring_kernel<false>);
    hipError_t e = set_lds(fn, lds);
    if (e != hipSuccess) return e;
    if (rows256)
      hipLaunchKernelGGL(vs_ring_kernel<true>, dim3(s.per_xcd * 8), dim3(256), lds, st, x, hl, v_idx, cover,
                         cover_bits, counts, nv, ns, cover_words, s);
    else
      hipLaunchKernelGGL(vs_ring_kernel<false>, dim3(s.per_xcd * 8), dim3(256), lds, st, x, hl, v_idx, cover,
                         cover_bits, counts, nv, ns, cover_words, s);
    return hipGetLastError();
  }
  const Sched s = make_sched(hl, x.group, NB);
  const size_t lds = 5 * HALF_BYTES;
  const void *fn = rows256 ? reinterpret_cast<const void *>(vs_kernel<true>)
                           : reinterpret_cast<const void *>(vs_kernel<false>);
  hipError_t e = set_lds(fn, lds);
  if (e != hipSuccess) return e;
  if (rows256)
    hipLaunchKernelGGL(vs_kernel<true>, dim3(s.per_xcd * 8), dim3(64), lds, st, x, hl, v_idx, cover, cover_bits,
                       counts, nv, ns, cover_words, s);
  else
    hipLaunchKernelGGL(vs_kernel<false>, dim3(s.per_xcd * 8), dim3(64), lds, st, x, hl, v_idx, cover, cover_bits,
                       counts, nv, ns, cover_words, s);
  return hipGetLastError();
}

hipError_t launch_vs_bs(const QKV &x, const HeadList &hv, const int32_t *v_idx, const int32_t *cover,
                        const uint32_t *cover_bits, const int32_t *counts, int nv, int ns, int cover_words,
                        const HeadList &hb, const int32_t *blk_idx, const int32_t *blk_cnt, const int32_t *order,
                        int topk, hipStream_t st) {
  const int NB = x.N / BQ;
  const Sched sv = make_sched(hv, x.group, NB), sb = make_sched(hb, x.group, NB);
  const VsArgs va{v_idx, cover, cover_bits, counts, nv, ns, cover_words};
  const BsArgs ba{blk_idx, blk_cnt, order, topk};
  const size_t lds = 5 * HALF_BYTES;
  const bool rows256 = x.k_st == D && x.v_st == D;
  const void *fn = rows256 ? reinterpret_cast<const void *>(vs_bs_kernel<true>)
                           : reinterpret_cast<const void *>(vs_bs_kernel<false>);
  hipError_t e = set_lds(fn, lds);
  if (e != hipSuccess) return e;
  // groups of 40 workgroup ids: 32 Vertical-Slash positions and 8 Block-Sparse positions
  const int groups = mixed_groups(sv, sb);
  if (rows256)
    hipLaunchKernelGGL(vs_bs_kernel<true>, dim3(40 * groups), dim3(64), lds, st, x, hv, va, sv, hb, ba, sb);
  else
    hipLaunchKernelGGL(vs_bs_kernel<false>, dim3(40 * groups), dim3(64), lds, st, x, hv, va, sv, hb, ba, sb);
  return hipGetLastError();
}

}  // namespace minf
