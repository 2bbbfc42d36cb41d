// Online sparse-index construction for gfx950 (MI355X).
//
// Vertical-Slash (Alg. 2, first steps; App. C.4.2):
//   A_hat = softmax(Q[-64:] K^T / sqrt(d) + causal), column sums, diagonal sums,
//   exact top-k of both, ascending sort, merge of the 64-wide slash tiles into
//   offset runs + a run bitmap.
//   K is streamed twice per K/V head (the query heads of a group share every K
//   tile): pass 1 gives the row max / row sum of the 64 estimating queries per
//   key chunk (combined afterwards in a fixed order), pass 2 forms the
//   normalised probabilities and reduces them along columns and diagonals.
//   A_hat itself (64 x N) is never stored.  All reductions run in a fixed
//   order: the scores are bit-reproducible.
//   Top-k of the line scores: an exact radix select on the order-preserving
//   integer image of the fp32 score (4 passes of 8 bits), ties to the lower
//   index, followed by an ordered compaction, so the kept indices come out
//   ascending without a sort.  From 128K scores on, a prefilter by many
//   workgroups (group maxima -> a lower bound of the k-th largest -> the scores
//   that reach it) leaves the select a few thousand candidates.
// Block-Sparse (Alg. 3, first steps):
//   mean pooling of Q and K over 64-token blocks (fp32); block logits with the
//   fp32 MFMA (the selection needs fp32-class logits) and the per-row top-k in
//   one kernel: candidate lists behind a rising bar, cut by bisection, exact
//   at the end; the logits are never stored.  Budgets above 112 blocks go
//   through stored logits and a per-row radix select.
#include <string.h>

#include "mfma_tile.h"

namespace minf {

typedef float f32x4v __attribute__((ext_vector_type(4)));

constexpr int VS_CHUNK = 1024;      // keys / offsets owned by one workgroup of the score kernels ...
constexpr int VS_CHUNK_SHORT = 256;  // ... for sequences up to VS_SHORT_N, where 1024 would leave most of the chip idle,
constexpr int VS_SHORT_N = 32768;
constexpr int VS_CHUNK_TINY = 128;   // ... and up to VS_TINY_N
constexpr int VS_TINY_N = 8192;

struct KvMap {                      // pooling work list of the Block-Sparse build
  int32_t n_kv;                     // distinct KV heads used by the call
  int32_t kv[MINF_MAX_HEADS];       // their ids
  int32_t slot_kv[MINF_MAX_HEADS];  // head slot -> position in kv[]
};

// Work list of the Vertical-Slash score kernels: the listed query heads grouped by the K/V
// head they read, at most four per group (one wave each).  The waves of a group share every K
// tile, so K is streamed once per group and pass instead of once per query head.
constexpr int VS_GROUP = 4;
struct VsGroups {
  int32_t n;                                  // groups
  uint8_t cnt[MINF_MAX_HEADS];                // query heads in the group (1 .. VS_GROUP)
  uint8_t slot[MINF_MAX_HEADS][VS_GROUP];     // their list slots
};

// ---------------------------------------------------------------------------
// helpers: order-preserving key, block-wide radix select, ordered compaction
// ---------------------------------------------------------------------------
__device__ inline unsigned order_key(float f) {
  unsigned u = __float_as_uint(f);
  return u ^ ((u >> 31) ? 0xffffffffu : 0x80000000u);
}

__device__ inline unsigned long long lanes_below(int lane) { return (1ull << lane) - 1ull; }

// Finds the k-th largest of data[0..n) (1 <= k <= n).  On return *thr is its
// key and *take_eq the number of elements equal to it that belong to the top-k
// (to be taken in index order).  hist: 256 ints of LDS, sh: 8 ints of LDS.
// VEC4: data is 16-byte aligned and n a multiple of 4; every thread then has
// eight elements (two 16-byte loads) in flight per round instead of one, which
// is what a single workgroup needs to stream a long row from memory.
template <int NT, bool VEC4>
__device__ inline void radix_select(const float *data, int n, int k, unsigned *thr, int *take_eq,
                                    int *hist, int *sh) {
  const int tid = threadIdx.x, lane = tid & 63;
  unsigned prefix = 0, mask = 0;
  int krem = k;
  for (int pass = 3; pass >= 0; --pass) {
    const int shift = 8 * pass;
    for (int i = tid; i < 256; i += NT) hist[i] = 0;
    __syncthreads();
    // one element per lane, wave-uniform control flow
    auto tally = [&](bool valid, unsigned u) {
      const bool part = valid && (u & mask) == prefix;
      const int d = (u >> shift) & 255;
      // Scores of one row often share their leading byte: add that byte's count
      // once per wave instead of 64 colliding LDS atomics.
      const unsigned long long bal = __builtin_amdgcn_ballot_w64(part);
      if (bal) {
        const int lead = __builtin_ctzll(bal);
        const int dl = __shfl(d, lead);
        const unsigned long long same = __builtin_amdgcn_ballot_w64(part && d == dl);
        if (lane == lead) atomicAdd(&hist[dl], __builtin_popcountll(same));
        if (part && d != dl) atomicAdd(&hist[d], 1);
      }
    };
    if (VEC4) {
      const float4 *d4 = reinterpret_cast<const float4 *>(data);
      const int n4 = n >> 2, n_round = (n4 + 2 * NT - 1) / (2 * NT) * (2 * NT);
      for (int i = tid; i < n_round; i += 2 * NT) {
        const bool v0 = i < n4, v1 = i + NT < n4;
        float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
        if (v0) a = d4[i];
        if (v1) b = d4[i + NT];
        tally(v0, order_key(a.x)); tally(v0, order_key(a.y)); tally(v0, order_key(a.z)); tally(v0, order_key(a.w));
        tally(v1, order_key(b.x)); tally(v1, order_key(b.y)); tally(v1, order_key(b.z)); tally(v1, order_key(b.w));
      }
    } else {
      const int n_round = (n + NT - 1) / NT * NT;
      for (int i = tid; i < n_round; i += NT) {
        const bool v = i < n;
        tally(v, v ? order_key(data[i]) : 0u);
      }
    }
    __syncthreads();
    // suffix sums over the 256 bins by the first 256 threads (4 waves)
    int suf = 0, own = 0;
    if (tid < 256) {
      own = hist[tid];
      suf = own;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_down(suf, off);
        if (lane + off < 64) suf += o;
      }
      if (lane == 0) sh[tid >> 6] = suf;      // wave totals
    }
    __syncthreads();
    if (tid < 256) {
      for (int w = (tid >> 6) + 1; w < 4; ++w) suf += sh[w];
      // suf = number of candidates with digit >= tid
      if (suf >= krem && suf - own < krem) {
        sh[4] = tid;
        sh[5] = krem - (suf - own);
      }
    }
    __syncthreads();
    prefix |= (unsigned)sh[4] << shift;
    mask |= 255u << shift;
    krem = sh[5];
    __syncthreads();
  }
  *thr = prefix;
  *take_eq = krem;
}

// Writes, ascending, the indices i with key(data[i]) > thr plus the first
// take_eq indices with key == thr.  Each wave owns a contiguous range; counts
// are exchanged through sh (2 * NT/64 ints of LDS).  VEC4 as above: a lane then
// holds four consecutive elements per 16-byte load, two loads in flight.
template <int NT, bool VEC4>
__device__ inline void ordered_select(const float *data, int n, unsigned thr, int take_eq, int32_t *out,
                                      int *sh, const int32_t *remap = nullptr) {
  // remap: the value written for element i is remap[i] instead of i (data is a compacted list)
  auto name_of = [&](int i) { return remap ? remap[i] : i; };
  constexpr int NW = NT / 64;
  constexpr int STEP = VEC4 ? 256 : 64;          // elements a wave takes per load
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int per = ((n + NW - 1) / NW + STEP - 1) / STEP * STEP;
  const int lo = min(wave * per, n), hi = min(lo + per, n);
  // keys of the elements a lane holds at position i0 of the wave's range (0 = below every score)
  auto load4 = [&](int i0, unsigned (&u)[4]) {
    const int i = i0 + 4 * lane;
    u[0] = u[1] = u[2] = u[3] = 0u;
    if (i < hi) {               // hi, lo and n are multiples of 4
      const float4 a = *reinterpret_cast<const float4 *>(data + i);
      u[0] = order_key(a.x); u[1] = order_key(a.y); u[2] = order_key(a.z); u[3] = order_key(a.w);
    }
  };
  int gt = 0, eq = 0;
  if (VEC4) {
    int g = 0, e = 0;
    for (int i0 = lo; i0 < hi; i0 += 2 * STEP) {
      unsigned u[4], w[4];
      load4(i0, u);
      load4(i0 + STEP, w);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        g += (u[c] > thr) + (w[c] > thr);
        e += (u[c] == thr && i0 + 4 * lane < hi) + (w[c] == thr && i0 + STEP + 4 * lane < hi);
      }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) { g += __shfl_xor(g, off); e += __shfl_xor(e, off); }
    gt = g; eq = e;
  } else {
    for (int i0 = lo; i0 < hi; i0 += 64) {
      const int i = i0 + lane;
      unsigned u = 0;
      const bool in = i < hi;
      if (in) u = order_key(data[i]);
      gt += __builtin_popcountll(__builtin_amdgcn_ballot_w64(in && u > thr));
      eq += __builtin_popcountll(__builtin_amdgcn_ballot_w64(in && u == thr));
    }
  }
  if (lane == 0) { sh[wave] = gt; sh[NW + wave] = eq; }
  __syncthreads();
  int pos = 0, eq_before = 0;
  for (int w = 0; w < wave; ++w) {
    const int e = sh[NW + w];
    pos += sh[w] + max(0, min(e, take_eq - eq_before));
    eq_before += e;
  }
  if (VEC4) {
    // one 256-element group: lane L holds elements 4L .. 4L+3 of it, in index order
    auto emit = [&](int i0, const unsigned (&u)[4]) {
      const bool in = i0 + 4 * lane < hi;
      int ne = 0, ns_ = 0;
      bool g[4], e[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) { g[c] = u[c] > thr; e[c] = in && u[c] == thr; ne += e[c]; }
      // equal elements before this lane's, in this group (exclusive lane scan)
      int e_scan = ne;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(e_scan, off);
        if (lane >= off) e_scan += o;
      }
      const int e_tot = __shfl(e_scan, 63);
      int rank = eq_before + e_scan - ne;
      bool sel[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        sel[c] = g[c] || (e[c] && rank < take_eq);
        rank += e[c];
        ns_ += sel[c];
      }
      int s_scan = ns_;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(s_scan, off);
        if (lane >= off) s_scan += o;
      }
      const int s_tot = __shfl(s_scan, 63);
      int p = pos + s_scan - ns_;
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (sel[c]) out[p++] = name_of(i0 + 4 * lane + c);
      pos += s_tot;
      eq_before += e_tot;
    };
    for (int i0 = lo; i0 < hi; i0 += 2 * STEP) {
      unsigned u[4], w[4];
      load4(i0, u);
      load4(i0 + STEP, w);
      // groups without a kept element (nearly all of a long row) cost two ballots
      bool any_u = false, any_w = false;
#pragma unroll
      for (int c = 0; c < 4; ++c) { any_u |= u[c] >= thr; any_w |= w[c] >= thr; }
      if (__builtin_amdgcn_ballot_w64(any_u)) emit(i0, u);
      if (__builtin_amdgcn_ballot_w64(any_w)) emit(i0 + STEP, w);
    }
  } else {
    for (int i0 = lo; i0 < hi; i0 += 64) {
      const int i = i0 + lane;
      unsigned u = 0;
      const bool in = i < hi;
      if (in) u = order_key(data[i]);
      const bool g = in && u > thr, e = in && u == thr;
      const unsigned long long eb = __builtin_amdgcn_ballot_w64(e);
      const int rank = eq_before + __builtin_popcountll(eb & lanes_below(lane));
      const bool sel = g || (e && rank < take_eq);
      const unsigned long long sb = __builtin_amdgcn_ballot_w64(sel);
      if (sel) out[pos + __builtin_popcountll(sb & lanes_below(lane))] = name_of(i);
      pos += __builtin_popcountll(sb);
      eq_before += __builtin_popcountll(eb);
    }
  }
  __syncthreads();
}

// k-th largest of n order keys held in LDS (1 <= k <= n); same contract as
// radix_select.  Meant for short lists: one key per thread and round.
template <int NT>
__device__ inline void radix_select_lds(const unsigned *keys, int n, int k, unsigned *thr, int *take_eq,
                                        int *hist, int *sh) {
  const int tid = threadIdx.x, lane = tid & 63;
  unsigned prefix = 0, mask = 0;
  int krem = k;
  for (int pass = 3; pass >= 0; --pass) {
    const int shift = 8 * pass;
    for (int i = tid; i < 256; i += NT) hist[i] = 0;
    __syncthreads();
    for (int i = tid; i < n; i += NT) {
      const unsigned u = keys[i];
      if ((u & mask) == prefix) atomicAdd(&hist[(u >> shift) & 255], 1);
    }
    __syncthreads();
    int suf = 0, own = 0;
    if (tid < 256) {
      own = hist[tid];
      suf = own;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_down(suf, off);
        if (lane + off < 64) suf += o;
      }
      if (lane == 0) sh[tid >> 6] = suf;
    }
    __syncthreads();
    if (tid < 256) {
      for (int w = (tid >> 6) + 1; w < 4; ++w) suf += sh[w];
      if (suf >= krem && suf - own < krem) {
        sh[4] = tid;
        sh[5] = krem - (suf - own);
      }
    }
    __syncthreads();
    prefix |= (unsigned)sh[4] << shift;
    mask |= 255u << shift;
    krem = sh[5];
    __syncthreads();
  }
  *thr = prefix;
  *take_eq = krem;
}

// Exclusive prefix sums of two counters over the 256 threads of a workgroup, in
// thread order; *ta, *tb receive the totals.  sh: 8 ints of LDS.
__device__ inline void block_scan2_256(int a, int b, int *ea, int *eb, int *ta, int *tb, int *sh) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int ia = a, ib = b;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int oa = __shfl_up(ia, off), ob = __shfl_up(ib, off);
    if (lane >= off) { ia += oa; ib += ob; }
  }
  if (lane == 63) { sh[wave] = ia; sh[4 + wave] = ib; }
  __syncthreads();
  int ba = 0, bb = 0, sa = 0, sb = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    if (w < wave) { ba += sh[w]; bb += sh[4 + w]; }
    sa += sh[w]; sb += sh[4 + w];
  }
  __syncthreads();
  *ea = ba + ia - a; *eb = bb + ib - b; *ta = sa; *tb = sb;
}

// ---------------------------------------------------------------------------
// Vertical-Slash score kernels.  Estimating row r (0..63) is query N-64+r; rows
// r < 64 - last_q do not take part.  Workgroup (group of query heads that read
// one K/V head, chunk c): four waves, one per query head of the group (a wave
// without a head only helps to fetch).  It owns the offsets [cC, cC+C) and the
// keys [N-cC-C, N-cC): tile m of the chunk holds the keys [N-cC-64(m+1),
// N-cC-64m); offsets of the chunk meet only tiles 0..C/64.  K tiles arrive by
// direct global -> LDS loads into three buffers (the swizzled layout of the
// attention kernels), a quarter per wave, the next tile in flight while the
// current one is reduced; one barrier per tile.  The tile is fetched once for
// the whole group: K is streamed once per K/V head and pass.
//  pass 1: S^T = K Q^T (keys along the accumulator registers): running row max
//          and row sum stay inside a lane.
//  pass 2: S = Q K^T (keys along the lanes, estimating rows along the
//          registers): a column sum is 32 in-lane adds and one exchange between
//          the lane halves.  For the diagonal sums the probabilities of 32 rows
//          go to LDS skewed, element (row, key) at column key - row + 32, so
//          that a diagonal is a column: every lane then adds up two columns.
//          Positions the skew never writes hold zeros from the start, so no
//          bounds are tested.  (LDS float atomics were tried for this and cost
//          about 700 cycles per instruction.)  One wave per head, program
//          order: the sums are reproducible.  The 64 x N estimate is never stored.
// ---------------------------------------------------------------------------
constexpr int VS_TILE_BYTES = TILE_BYTES;          // 16 KiB
constexpr int VS_DPAD = 96;                       // slack on both sides of the chunk's diagonal sums
constexpr int VS_SKEW_PITCH = 64;                 // floats per row of the skewed probability tile (32 rows x 32 keys)
constexpr int vs_wave_floats(int C) { return C + 2 * VS_DPAD + 32 * VS_SKEW_PITCH; }   // pass 2, private to a wave

// This wave's quarter of a K tile of ROWS rows (64 or 32) that lies wholly inside [0, N).
template <int ROWS>
__device__ inline void vs_fetch_quarter(const bf16_t *kh, int64_t k_st, const DmaLane &dl, int kbase, char *tile,
                                        int wave) {
  constexpr int PER = ROWS / 4 / VS_GROUP;          // 1 KiB blocks per wave: 4 or 2
  const bf16_t *ubase = kh + (int64_t)kbase * k_st;
  const unsigned base = lds_addr_of(tile);
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int blk = wave * PER + i;
    // block blk takes the lane offsets of blk % 4: i for whole groups of four, 2 (wave % 2) + i for pairs
    const unsigned voff = PER == 4 ? dl.voff[i] : ((wave & 1) ? dl.voff[2 + i] : dl.voff[i]);
    dma16_su(ubase + (int64_t)(4 * blk) * k_st, voff, base + blk * 1024);
  }
}

// Adds the diagonal sums of a 32 x 32 tile of probabilities to dbase[-63 .. 0].  p[r] is the
// element (local row rl = 8 (r / 4) + 4 h + r % 4, key column n) of this lane (n = lane % 32,
// h = lane / 32).  The tile goes to LDS skewed, element (rl, n) at column n - rl + 32, so that a
// diagonal is a column; column j belongs to dbase[-j].  Lane (cp = n, rh = h) then adds up the
// columns 2 cp, 2 cp + 1 over the rows 16 rh .. 16 rh + 15 (8-byte reads) and the two row halves
// meet in the lanes rh = 0.  Positions the skew never writes hold zeros from the start.  One wave,
// program order: reproducible.
__device__ inline void vs_skew_reduce(const float (&p)[16], float *skew, float *dbase, int n, int h) {
  float *wlane = skew + 4 * h * (VS_SKEW_PITCH - 1) + n + 32;
#pragma unroll
  for (int r = 0; r < 16; ++r) wlane[(8 * (r >> 2) + (r & 3)) * (VS_SKEW_PITCH - 1)] = p[r];
  // (LDS operations of one wave execute in order; the fences are for the compiler)
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  const float2 *col2 = reinterpret_cast<const float2 *>(skew + 16 * h * VS_SKEW_PITCH) + n;
  float t0 = 0.f, t1 = 0.f;
#pragma unroll
  for (int rl = 0; rl < 16; ++rl) {
    const float2 e = col2[rl * (VS_SKEW_PITCH / 2)];
    t0 += e.x;
    t1 += e.y;
  }
  const float u0 = __shfl_xor(t0, 32), u1 = __shfl_xor(t1, 32);
  if (h == 0) {
    dbase[-2 * n] += t0 + u0;          // column 2 n
    dbase[-2 * n - 1] += t1 + u1;      // column 2 n + 1
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int PASS, int C>
__global__ __launch_bounds__(256, 2) void vs_score_kernel(QKV x, HeadList hl, VsGroups vg, int last_q, int n_chunks,
                                                       float *ml_part, const float *ml_fin,
                                                       float *colsum, float *diagsum) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  // pass 1: three shared 64-key K tiles.  pass 2: three shared 32-key K half tiles, then per wave
  // the diagonal sums and the skewed tile.
  const int grp = blockIdx.y, chunk = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool active = wave < vg.cnt[grp];
  // a wave without a head takes the group's first one for its addresses; it only helps to fetch
  const int slot = __builtin_amdgcn_readfirstlane((int)vg.slot[grp][active ? wave : 0]);
  float *dacc = reinterpret_cast<float *>(lds + 3 * HALF_BYTES) + wave * vs_wave_floats(C);   // [VS_DPAD + C + VS_DPAD], pass 2
  float *skew = dacc + C + 2 * VS_DPAD;                                // [32][VS_SKEW_PITCH], pass 2

  const int head = __builtin_amdgcn_readfirstlane(hl.h[slot]);
  const int kvh = to_sgpr(head / x.group);
  const bf16_t *qh = x.q + head * x.q_sh, *kh = x.k + kvh * x.k_sh;
  const int n = lane & 31, h = lane >> 5;
  const int N = x.N;
  const int r_min = 64 - last_q;

  // Q fragments: lane (n, h) holds Q[N-64 + 32 nb + n][16 ks + 8 h .. +7], which is the B operand
  // of K Q^T and the A operand of Q K^T alike
  bf16x8 q[2][8];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    const bf16_t *row = qh + (int64_t)(N - 64 + 32 * nb + n) * x.q_st + 8 * h;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) q[nb][ks] = *reinterpret_cast<const bf16x8 *>(row + 16 * ks);
  }
  LaneOfs lo;
  lane_offsets(lo, lane);
  DmaLane dl;
  dma_lane_init(dl, x.k_st, lane);

  // pass 1 state: lane (n, h) follows rows 32 nb + n over its half of the keys
  float m_run0 = -INFINITY, m_run1 = -INFINITY, l_run0 = 0.f, l_run1 = 0.f;
  // pass 2: per register of the S layout, row 32 nb + 8 (r / 4) + 4 h + r % 4 needs its
  // exponent offset  max + log2(sum)  (+inf for a row that does not take part: P = 0)
  float off[2][16];
  if (PASS == 2) {
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = 32 * nb + 8 * (r >> 2) + 4 * h + (r & 3);
        const float mx = ml_fin[(slot * 64 + row) * 2 + 0], inv = ml_fin[(slot * 64 + row) * 2 + 1];
        off[nb][r] = (row >= r_min && inv > 0.f) ? mx - __builtin_amdgcn_logf(inv) : INFINITY;
      }
    for (int i = lane; i < C + 2 * VS_DPAD + 32 * VS_SKEW_PITCH; i += 64) dacc[i] = 0.f;   // dacc and skew
    __syncthreads();
  }

  const int key_hi = N - chunk * C;                 // exclusive end of the owned keys

  if (PASS == 1) {
    // 64-key tiles, two 16 KiB buffers; tiles are 64-aligned: wholly inside [0, N) or outside
    const int n_tiles = min(C / 64, key_hi / 64);
    auto tile_key = [&](int mm) { return key_hi - 64 * (mm + 1); };
    // three buffers, two tiles in flight: tile i lives in buffer i mod 3
    auto fetch = [&](int mm) {
      vs_fetch_quarter<64>(kh, x.k_st, dl, tile_key(mm), lds + (mm % 3) * VS_TILE_BYTES, wave);
    };
    if (n_tiles > 0) fetch(0);
    if (n_tiles > 1) fetch(1);
    for (int m = 0; m < n_tiles; ++m) {
      const int kt = tile_key(m);
      const char *tK = lds + (m % 3) * VS_TILE_BYTES;
      // Tile m has landed once every wave has waited for its quarter (its own four loads of tile
      // m+1 may stay in flight).  Behind the barrier every wave is also done with tile m-1, whose
      // buffer the fetch of tile m+2 overwrites.
      if (m + 1 < n_tiles) MINF_WAIT_VMCNT(4); else MINF_WAIT_VMCNT(0);
      __syncthreads();
      if (m + 2 < n_tiles) fetch(m + 2);
      if (!active) continue;                         // a wave without a head only fetches
      const bool diag_tile = kt + 63 > N - 64;       // only the last 64 keys are cut by causality
      f32x16 s[2][2];
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) s[i][j][r] = 0.f;
      // s[mb][nb]: register e holds key kt + 32 mb + 16 (e / 8) + 8 h + e % 8, row 32 nb + n
#pragma unroll
      for (int ks = 0; ks < 8; ++ks)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
          const bf16x8 a = lds_read_k(tK, lo.k[ks] + mb * HALF_BYTES);
          s[mb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, q[0][ks], s[mb][0], 0, 0, 0);
          s[mb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, q[1][ks], s[mb][1], 0, 0, 0);
        }
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        float &m_run = nb == 0 ? m_run0 : m_run1;
        float &l_run = nb == 0 ? l_run0 : l_run1;
        if (!diag_tile && r_min == 0) {
          // no element of the tile is masked (all but the last tile of a head): the maximum is
          // taken over the raw logits and the scale rides in the exponent's multiply-add
          float mx = s[0][nb][0];
#pragma unroll
          for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[mb][nb][e]);
          const float m_new = fmaxf(m_run, mx * x.c_log2);
          float sum = 0.f;
#pragma unroll
          for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int e = 0; e < 16; ++e) sum += fast_exp2(fmaf(s[mb][nb][e], x.c_log2, -m_new));
          l_run = l_run * fast_exp2(m_run - m_new) + sum;
          m_run = m_new;
          continue;
        }
        const int r = 32 * nb + n, p = N - 64 + r;
        float mx = -INFINITY;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            float v = s[mb][nb][e] * x.c_log2;
            if (diag_tile) {
              const int key = kt + 32 * mb + 16 * (e >> 3) + 8 * h + (e & 7);
              v = key <= p ? v : -INFINITY;
            }
            v = r >= r_min ? v : -INFINITY;
            s[mb][nb][e] = v;
            mx = fmaxf(mx, v);
          }
        const float m_new = fmaxf(m_run, mx);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        float sum = 0.f;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int e = 0; e < 16; ++e) sum += fast_exp2(s[mb][nb][e] - m_use);
        l_run = l_run * fast_exp2(m_run - m_use) + sum;
        m_run = m_new;
      }
    }
  } else {
    // 32-key half tiles, two 8 KiB buffers.  The offsets of the chunk meet the half tiles
    // 0 .. C/32 + 1; the chunk's own keys are the half tiles 0 .. C/32 - 1.
    const int n_half = min(C / 32 + 2, key_hi / 32);
    auto tile_key = [&](int mm) { return key_hi - 32 * (mm + 1); };
    auto fetch = [&](int mm) {
      vs_fetch_quarter<32>(kh, x.k_st, dl, tile_key(mm), lds + (mm % 3) * HALF_BYTES, wave);
    };
    // lane (n, h) reads K row n of the half tile: keys run along the lanes in index order
    int kofs[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) kofs[ks] = swz_byte(n, 2 * ks + h);
    float carry[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) carry[r] = 0.f;
    if (n_half > 0) fetch(0);
    if (n_half > 1) fetch(1);
    for (int m = 0; m < n_half; ++m) {
      const int kt = tile_key(m);
      const char *tK = lds + (m % 3) * HALF_BYTES;
      // As in pass 1: three buffers, one barrier per half tile.  At most the two youngest memory
      // operations of this wave may stay in flight; whatever they are (the two loads of half tile
      // m+1, or one of them and the column-sum store of the iteration before), half tile m is
      // older and has landed.
      if (m + 1 < n_half) MINF_WAIT_VMCNT(2); else MINF_WAIT_VMCNT(0);
      __syncthreads();
      if (m + 2 < n_half) fetch(m + 2);
      if (!active) continue;
      const bool diag_tile = kt + 31 > N - 64;
      // s[nb]: register r holds row 32 nb + 8 (r / 4) + 4 h + r % 4, key kt + n
      f32x16 s[2];
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[j][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 kf = lds_read_k(tK, kofs[ks]);
        s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q[0][ks], kf, s[0], 0, 0, 0);
        s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q[1][ks], kf, s[1], 0, 0, 0);
      }
      // probabilities of the half tile: pv[nb][r] for row 32 nb + 8 (r / 4) + 4 h + r % 4, key kt + n
      float pv[2][16];
      float cs = 0.f;
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) pv[nb][r] = fast_exp2(fmaf(s[nb][r], x.c_log2, -off[nb][r]));
        if (diag_tile) {           // only the last two half tiles of a head are cut by causality
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int rl4 = 8 * (r >> 2) + (r & 3);                    // local row - 4 h
            pv[nb][r] = kt + n <= N - 64 + 32 * nb + rl4 + 4 * h ? pv[nb][r] : 0.f;
          }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) cs += pv[nb][r];
      }
      // Diagonal sums.  Element (row 32 + rl, key kt + n) of this half tile and element (row rl,
      // key kt - 32 + n) of the next one lie on the same diagonal and in the same register and
      // lane, so the upper 32 rows wait one iteration (carry) and go through LDS together with the
      // lower 32 rows of the next half tile: one skewed tile per half tile instead of two.
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float both = pv[0][r] + carry[r];
        carry[r] = pv[1][r];
        pv[0][r] = both;
      }
      vs_skew_reduce(pv[0], skew, dacc + VS_DPAD + 32 * m, n, h);
      // the two lane halves hold the two halves of the rows of the same key
      const float other = __shfl_xor(cs, 32);
      const float tot = h == 0 ? cs + other : other + cs;   // same operand order in both
      if (active && h == 0 && m < C / 32) colsum[(int64_t)slot * N + kt + n] = tot;
    }
    // the upper rows of the last half tile
    vs_skew_reduce(carry, skew, dacc + VS_DPAD + 32 * n_half, n, h);
  }

  if (PASS == 1) {
    // merge the two lanes that share an estimating row, store the chunk's (max, sum)
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const float m_run = nb == 0 ? m_run0 : m_run1, l_run = nb == 0 ? l_run0 : l_run1;
      const float mo = __shfl_xor(m_run, 32), lo2 = __shfl_xor(l_run, 32);
      const float M = fmaxf(m_run, mo);
      const float Mu = M == -INFINITY ? 0.f : M;
      // same operand order in both lanes of the pair: lane-half 0's share first
      const float a = h == 0 ? l_run * fast_exp2(m_run - Mu) : lo2 * fast_exp2(mo - Mu);
      const float b = h == 0 ? lo2 * fast_exp2(mo - Mu) : l_run * fast_exp2(m_run - Mu);
      if (active && h == 0) {
        float *dst = ml_part + (((int64_t)slot * n_chunks + chunk) * 64 + 32 * nb + n) * 2;
        dst[0] = M;
        dst[1] = a + b;
      }
    }
  } else {
    __syncthreads();
    for (int i = lane; i < C; i += 64) {
      const int o = chunk * C + i;
      if (active && o < N) diagsum[(int64_t)slot * N + o] = dacc[VS_DPAD + i];
    }
  }
}

// Combine the per-chunk (max, sum) pairs of every estimating row into (row max,
// 1 / row sum).  16 waves per head: wave g reduces a contiguous range of chunks
// in chunk order, the 16 partial results are then combined in wave order, so the
// result does not depend on timing.
__global__ __launch_bounds__(1024) void vs_combine_kernel(int n_chunks, const float *ml_part, float *ml_fin) {
  __shared__ float red[16][64];
  const int slot = blockIdx.x, r = threadIdx.x & 63, g = threadIdx.x >> 6;
  const float2 *src = reinterpret_cast<const float2 *>(ml_part) + (int64_t)slot * n_chunks * 64 + r;
  const int per = (n_chunks + 15) / 16, c0 = min(g * per, n_chunks), c1 = min(c0 + per, n_chunks);
  float M = -INFINITY;
#pragma unroll 8
  for (int c = c0; c < c1; ++c) M = fmaxf(M, src[c * 64].x);
  red[g][r] = M;
  __syncthreads();
  M = red[0][r];
#pragma unroll
  for (int i = 1; i < 16; ++i) M = fmaxf(M, red[i][r]);
  __syncthreads();
  float L = 0.f;
  if (M != -INFINITY) {
#pragma unroll 8
    for (int c = c0; c < c1; ++c) {
      const float2 ml = src[c * 64];
      L += ml.y * fast_exp2(ml.x - M);
    }
  }
  red[g][r] = L;
  __syncthreads();
  if (g == 0) {
    L = red[0][r];
#pragma unroll
    for (int i = 1; i < 16; ++i) L += red[i][r];
    ml_fin[(slot * 64 + r) * 2 + 0] = M == -INFINITY ? 0.f : M;
    ml_fin[(slot * 64 + r) * 2 + 1] = L > 0.f ? 1.0f / L : 0.f;
  }
}

// "sparseformat" (Alg. 2; the role of Alg. 4, App. C.4.2): the ascending kept slash offsets
// offs[0 .. k) of one head become offset runs [t0, t1) -- slash o covers the offsets (o - 64, o],
// the 64 x 64 tile whose main diagonal it is; neighbours at most 64 apart merge -- and the run
// bitmap (bit t + 64 set iff offset t is covered).  1024 threads; sh: 16 ints of LDS.  Returns the
// number of runs.  Offsets are clamped into [0, N), so that a list the caller filled badly cannot
// make the bitmap writes leave the head's words.
__device__ inline int vs_merge_runs(const int32_t *offs, int k, int N, int2 *runs, uint32_t *bits,
                                    int cover_words, int *sh) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < cover_words; i += 1024) bits[i] = 0u;
  __threadfence_block();
  __syncthreads();
  auto at = [&](int i) { return min(max(offs[i], 0), N - 1); };
  int run_base = 0;
  // ---- a gap of more than 64 between neighbouring kept offsets ends a run
  for (int i0 = 0; i0 < k; i0 += 1024) {
    const int i = i0 + tid;
    int o = 0;
    bool start = false, last = false;
    if (i < k) {
      o = at(i);
      start = i == 0 || o - at(i - 1) > 64;
      last = i == k - 1 || at(i + 1) - o > 64;
    }
    const unsigned long long sb = __builtin_amdgcn_ballot_w64(start);
    if (lane == 0) sh[wave] = __builtin_popcountll(sb);
    __syncthreads();
    int before = run_base, total = 0;
    for (int w = 0; w < 16; ++w) {
      const int c = sh[w];
      if (w < wave) before += c;
      total += c;
    }
    // run id of element i = (number of starts at or before i) - 1
    const int rid = before + __builtin_popcountll(sb & lanes_below(lane)) + (start ? 1 : 0) - 1;
    if (start) runs[rid].x = o - 63;
    if (last) runs[rid].y = o + 1;
    run_base += total;
    __syncthreads();
  }
  // ---- run bitmap: run [t0, t1) sets the bits t0 + 64 .. t1 + 63, one wave per run, one lane per
  // word.  Runs are disjoint, so only the first and the last word of a run can be shared with a
  // neighbour and need an atomic; the words in between are whole.  (One atomic per kept offset
  // and word, as a first version had it, makes thousands of atomics meet on the same few words.)
  __threadfence_block();
  __syncthreads();
  for (int r = wave; r < run_base; r += 16) {
    const int2 rr = runs[r];
    const int b0 = rr.x + 64, b1 = rr.y + 63;          // inclusive bit range
    const int w0 = b0 >> 5, w1 = b1 >> 5;
    for (int w = w0 + lane; w <= w1; w += 64) {
      unsigned m = 0xffffffffu;
      if (w == w0) m &= ~((1u << (b0 & 31)) - 1u);
      if (w == w1 && (b1 & 31) != 31) m &= (1u << ((b1 & 31) + 1)) - 1u;
      if (w == w0 || w == w1) atomicOr(&bits[w], m);
      else bits[w] = m;
    }
  }
  return run_base;
}

// ---------------------------------------------------------------------------
// Prefilter of the line-score top-k (Alg. 2: top-k of the column sums and of the
// diagonal sums).  One workgroup streaming a 4 MiB row six times is bound by
// latency, so the long rows are cut down first by many workgroups:
//   vs_gmax_kernel    maximum of every group of G consecutive scores (G a power of two with
//                     N / G >= 4 k);
//   vs_bound_kernel   the k-th largest group maximum: k different scores reach it, so it is a
//                     lower bound of the k-th largest score, and every score of the top-k set
//                     (ties included) reaches it too;
//   vs_filter_kernel  the scores that reach the bound, with their positions, compacted slice by
//                     slice (in position order inside a slice; slices take their room from a
//                     counter in arrival order and record where they put their part);
//   vs_select_kernel  puts the parts in slice order and runs the exact selection on the
//                     candidates (about 0.3 N / G of them) instead of the row.
// If the candidates do not fit their buffer (plateaus of equal scores) or no G in 4 .. 64
// satisfies N / G >= 4 k, vs_select_kernel selects from the whole row as before.  The result is
// the same in both cases: exact top-k, equal scores to the lower position.
// ---------------------------------------------------------------------------
constexpr int VS_SLICE = 16384;                     // scores per workgroup of the filter
struct VsSelState {                                 // per (head slot, which), in the workspace
  unsigned bound;                                   // order key of the lower bound
  int count;                                        // candidates taken so far (room counter)
  int overflow;                                     // some slice found no room
  int log_g;                                        // log2 G, or -1: no prefilter for this row
};

__device__ inline float key_to_float(unsigned key) {
  return __uint_as_float((key & 0x80000000u) ? key ^ 0x80000000u : ~key);
}

// largest G = 2^g, 2 <= g <= 6, with N / G >= 4 k; -1 if there is none, or if the row is so short
// that the three extra launches cost more than they save (below 128K scores)
inline int vs_log_group(int N, int k) {
  if (N < 131072) return -1;
  for (int g = 6; g >= 2; --g)
    if ((int64_t)(N >> g) >= 4 * (int64_t)k) return g;
  return -1;
}

// grid (ceil(N / 4096), heads, 2), 256 threads: thread t of a workgroup holds the scores
// 4 (256 j + t) .. + 3 of its 4096; a group of G scores is G / 4 neighbouring lanes.
__global__ __launch_bounds__(256) void vs_gmax_kernel(int N, int log_gv, int log_gs, const float *colsum,
                                                      const float *diagsum, float *gmax_v, float *gmax_s) {
  const int slot = blockIdx.y, which = blockIdx.z;
  const int log_g = which == 0 ? log_gv : log_gs;
  if (log_g < 0) return;
  const float *data = (which == 0 ? colsum : diagsum) + (int64_t)slot * N;
  float *gm = (which == 0 ? gmax_v : gmax_s) + (int64_t)slot * (N >> 2);
  const int lanes = 1 << (log_g - 2);               // lanes per group
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int i = blockIdx.x * 4096 + (j * 256 + threadIdx.x) * 4;
    unsigned m = 0u;                                 // below every key
    if (i < N) {
      const float4 a = *reinterpret_cast<const float4 *>(data + i);
      m = max(max(order_key(a.x), order_key(a.y)), max(order_key(a.z), order_key(a.w)));
    }
    for (int off = 1; off < lanes; off <<= 1) m = max(m, (unsigned)__shfl_xor((int)m, off));
    if (i < N && (threadIdx.x & (lanes - 1)) == 0) gm[i >> log_g] = key_to_float(m);
  }
}

// grid (heads, 2), 1024 threads
__global__ __launch_bounds__(1024) void vs_bound_kernel(int N, int nv, int ns, int log_gv, int log_gs,
                                                        const float *gmax_v, const float *gmax_s,
                                                        VsSelState *state) {
  __shared__ int hist[256];
  __shared__ int sh[16];
  const int slot = blockIdx.x, which = blockIdx.y;
  const int log_g = which == 0 ? log_gv : log_gs;
  VsSelState *st = state + slot * 2 + which;
  unsigned thr = 0u;
  if (log_g >= 0) {
    const float *gm = (which == 0 ? gmax_v : gmax_s) + (int64_t)slot * (N >> 2);
    const int n_g = N >> log_g, k = min(which == 0 ? nv : ns, N);
    int take_eq;
    if ((n_g & 3) == 0) radix_select<1024, true>(gm, n_g, k, &thr, &take_eq, hist, sh);
    else radix_select<1024, false>(gm, n_g, k, &thr, &take_eq, hist, sh);
  }
  if (threadIdx.x == 0) {
    st->bound = thr;
    st->count = 0;
    st->overflow = 0;
    st->log_g = log_g;
  }
}

// grid (ceil(N / VS_SLICE), heads, 2), 256 threads.  Wave w of a workgroup owns the scores
// 4096 w .. 4096 w + 4095 of the slice, 256 at a time (lane L: 4 L .. 4 L + 3), held in registers.
__global__ __launch_bounds__(256) void vs_filter_kernel(int N, int cap, int n_slices, const float *colsum,
                                                        const float *diagsum, VsSelState *state,
                                                        float *cand_val, int32_t *cand_idx, int2 *seg) {
  __shared__ int sh[8];
  const int sl = blockIdx.x, slot = blockIdx.y, which = blockIdx.z;
  VsSelState *st = state + slot * 2 + which;
  int2 *myseg = seg + ((int64_t)(slot * 2 + which)) * n_slices + sl;
  if (st->log_g < 0) return;
  const unsigned bound = st->bound;
  const float *data = (which == 0 ? colsum : diagsum) + (int64_t)slot * N;
  float *cv = cand_val + (int64_t)(slot * 2 + which) * cap;
  int32_t *ci = cand_idx + (int64_t)(slot * 2 + which) * cap;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int w0 = sl * VS_SLICE + wave * 4096;
  float4 v[16];
  int mine = 0;
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const int i = w0 + j * 256 + 4 * lane;
    v[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < N) {                                     // N is a multiple of 4
      v[j] = *reinterpret_cast<const float4 *>(data + i);
      mine += (order_key(v[j].x) >= bound) + (order_key(v[j].y) >= bound) + (order_key(v[j].z) >= bound) +
              (order_key(v[j].w) >= bound);
    }
  }
  // candidates of the waves before this one, and of the slice
  int wsum = mine;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) wsum += __shfl_xor(wsum, off);
  if (lane == 0) sh[wave] = wsum;
  __syncthreads();
  const int total = sh[0] + sh[1] + sh[2] + sh[3];
  if (tid == 0) {
    int base = 0;
    if (total > 0) {
      base = atomicAdd(&st->count, total);
      if (base + total > cap) {
        atomicExch(&st->overflow, 1);
        base = -1;
      }
    }
    sh[4] = base;
    *myseg = make_int2(base, total);
  }
  __syncthreads();
  const int base = sh[4];
  if (total == 0 || base < 0) return;
  int pos = base;
  for (int w = 0; w < wave; ++w) pos += sh[w];
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const int i = w0 + j * 256 + 4 * lane;
    const float e[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
    bool take[4];
    int n_take = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      take[c] = i < N && order_key(e[c]) >= bound;
      n_take += take[c];
    }
    if (__builtin_amdgcn_ballot_w64(n_take > 0) == 0) continue;      // wave-uniform
    int scan = n_take;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int o = __shfl_up(scan, off);
      if (lane >= off) scan += o;
    }
    int p = pos + scan - n_take;
#pragma unroll
    for (int c = 0; c < 4; ++c)
      if (take[c]) {
        cv[p] = e[c];
        ci[p] = i + c;
        ++p;
      }
    pos += __shfl(scan, 63);
  }
}

// Top-k + "sparseformat".  blockIdx.y = 0: verticals from the column sums;
// blockIdx.y = 1: slashes from the diagonal sums, their runs and the run bitmap.
__global__ __launch_bounds__(1024) void vs_select_kernel(int N, int nv, int ns, const float *colsum,
                                                         const float *diagsum, int32_t *v_idx,
                                                         int32_t *s_idx, int32_t *cover,
                                                         uint32_t *cover_bits, int32_t *counts,
                                                         int cover_words, int cap, int n_slices,
                                                         const VsSelState *state, const float *cand_val,
                                                         const int32_t *cand_idx, const int2 *seg,
                                                         float *list_val, int32_t *list_idx) {
  __shared__ int hist[256];
  __shared__ int sh[40];
  __shared__ int seg_pos[256];
  const int slot = blockIdx.x, which = blockIdx.y, tid = threadIdx.x;
  const float *data = (which == 0 ? colsum : diagsum) + (int64_t)slot * N;
  const int kcap = which == 0 ? nv : ns;
  const int k = min(kcap, N);
  int32_t *out = which == 0 ? v_idx + (int64_t)slot * nv : s_idx + (int64_t)slot * ns;
  unsigned thr;
  int take_eq;
  // n_slices == 0: the launch ran no prefilter (the state was not written)
  VsSelState st;
  st.bound = 0u; st.count = 0; st.overflow = 1; st.log_g = -1;
  if (n_slices > 0) st = state[slot * 2 + which];
  // the prefilter's candidates are complete (every slice found room) and in use for this row
  const bool filtered = st.log_g >= 0 && st.overflow == 0 && st.count >= k && st.count <= cap && n_slices <= 256;
  if (filtered) {
    // the slices' parts, in slice order, into one list (position order)
    const int2 *sg = seg + (int64_t)(slot * 2 + which) * n_slices;
    if (tid == 0) {
      int p = 0;
      for (int i = 0; i < n_slices; ++i) {
        seg_pos[i] = p;
        p += sg[i].y;
      }
    }
    __syncthreads();
    const float *cv = cand_val + (int64_t)(slot * 2 + which) * cap;
    const int32_t *ci = cand_idx + (int64_t)(slot * 2 + which) * cap;
    float *lv = list_val + (int64_t)(slot * 2 + which) * cap;
    int32_t *li = list_idx + (int64_t)(slot * 2 + which) * cap;
    const int wave = tid >> 6, lane = tid & 63;
    for (int i = wave; i < n_slices; i += 16) {
      const int2 g = sg[i];
      for (int e = lane; e < g.y; e += 64) {
        lv[seg_pos[i] + e] = cv[g.x + e];
        li[seg_pos[i] + e] = ci[g.x + e];
      }
    }
    __threadfence_block();
    __syncthreads();
    radix_select<1024, false>(lv, st.count, k, &thr, &take_eq, hist, sh);
    ordered_select<1024, false>(lv, st.count, thr, take_eq, out, sh + 8, li);
  } else {
    radix_select<1024, true>(data, N, k, &thr, &take_eq, hist, sh);      // N % 64 == 0, rows 256-byte aligned
    ordered_select<1024, true>(data, N, thr, take_eq, out, sh + 8);
  }
  for (int i = k + tid; i < kcap; i += 1024) out[i] = 0;
  if (which == 0) {
    if (tid == 0) counts[slot * 4 + 0] = k;
    return;
  }
  const int n_runs = vs_merge_runs(out, k, N, reinterpret_cast<int2 *>(cover) + (int64_t)slot * ns,
                                   cover_bits + (int64_t)slot * cover_words, cover_words, sh + 8);
  if (tid == 0) {
    counts[slot * 4 + 1] = k;
    counts[slot * 4 + 2] = n_runs;
    counts[slot * 4 + 3] = 0;
  }
}

// "sparseformat" alone, for lines the caller supplies (the static-index use of the attention
// call): one workgroup per head builds runs, bitmap and the run count from s_idx[0 .. n_s).
__global__ __launch_bounds__(1024) void vs_lines_kernel(int N, int nv, int ns, const int32_t *s_idx,
                                                        int32_t *cover, uint32_t *cover_bits,
                                                        int32_t *counts, int cover_words) {
  __shared__ int sh[24];
  const int slot = blockIdx.x;
  const int n_v = min(max(counts[slot * 4 + 0], 0), nv), n_s = min(max(counts[slot * 4 + 1], 0), ns);
  __syncthreads();           // every thread has read the counts before thread 0 rewrites them
  const int n_runs = vs_merge_runs(s_idx + (int64_t)slot * ns, n_s, N,
                                   reinterpret_cast<int2 *>(cover) + (int64_t)slot * ns,
                                   cover_bits + (int64_t)slot * cover_words, cover_words, sh);
  if (threadIdx.x == 0) {
    counts[slot * 4 + 0] = n_v;
    counts[slot * 4 + 1] = n_s;
    counts[slot * 4 + 2] = n_runs;
    counts[slot * 4 + 3] = 0;
  }
}

// ---------------------------------------------------------------------------
// Block-Sparse: pooling, block logits, per-row top-k
// ---------------------------------------------------------------------------
// grid (NB, n_heads + n_kv): y < n_heads pools Q of head slot y, else K of kv[y - n_heads]
// (the pooled K vectors of a K/V head are NBp >= NB rows apart: padded to whole 32-row tiles)
// grid (NB, n_q + n_kv): n_q = the listed query heads, or 0 (qpool == nullptr) when the caller pools Q itself.
__global__ __launch_bounds__(256) void bs_pool_kernel(QKV x, HeadList hl, KvMap km, float *qpool, float *kpool,
                                                      int NBp) {
  __shared__ float red[16][132];
  const int b = blockIdx.x, NB = x.N / 64;
  const int y = qpool ? blockIdx.y : blockIdx.y + hl.n;
  const bf16_t *src;
  int64_t st;
  float *dst;
  if (y < hl.n) {
    src = x.q + hl.h[y] * x.q_sh; st = x.q_st; dst = qpool + ((int64_t)y * NB + b) * 128;
  } else {
    src = x.k + km.kv[y - hl.n] * x.k_sh; st = x.k_st; dst = kpool + ((int64_t)(y - hl.n) * NBp + b) * 128;
  }
  const int tid = threadIdx.x, r = tid >> 4, c = tid & 15;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint4 w = *reinterpret_cast<const uint4 *>(src + (int64_t)(b * 64 + r + 16 * i) * st + c * 8);
    const unsigned ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      acc[2 * j] += __uint_as_float(ww[j] << 16);
      acc[2 * j + 1] += __uint_as_float(ww[j] & 0xffff0000u);
    }
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) red[r][c * 8 + j] = acc[j];
  __syncthreads();
  if (tid < 128) {
    float s = 0.f;
#pragma unroll
    for (int rr = 0; rr < 16; ++rr) s += red[rr][tid];
    dst[tid] = s * (1.0f / 64.0f);
  }
}

// Block logits of the lower triangle, one wave per 64 x 64 tile, fp32 MFMA
// (v_mfma_f32_32x32x2_f32).  grid (tiles of the lower triangle, heads of the batch).
__global__ __launch_bounds__(64) void bs_logits_kernel(int NB, int NBp, int slot0, KvMap km, const float *qpool,
                                                       const float *kpool, float *scores, float scale) {
  const int t = blockIdx.x, hb = blockIdx.y, slot = slot0 + hb;
  // t -> (ti, tj), tj <= ti
  int ti = (int)((sqrtf(8.0f * (float)t + 1.0f) - 1.0f) * 0.5f);
  while ((ti + 1) * (ti + 2) / 2 <= t) ++ti;
  while (ti * (ti + 1) / 2 > t) --ti;
  const int tj = t - ti * (ti + 1) / 2;
  const int lane = threadIdx.x, n = lane & 31, h = lane >> 5;
  const float *qp = qpool + (int64_t)slot * NB * 128;
  const float *kp = kpool + (int64_t)km.slot_kv[slot] * NBp * 128;
  f32x16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
  const float *arow[2], *brow[2];
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    arow[a] = qp + (int64_t)min(ti * 64 + 32 * a + n, NB - 1) * 128 + 8 * h;
    brow[a] = kp + (int64_t)min(tj * 64 + 32 * a + n, NB - 1) * 128 + 8 * h;
  }
  // contraction index of step (ch, i): d = 16ch + 8h + i, the same for both operands
#pragma unroll 2
  for (int ch = 0; ch < 8; ++ch) {
    float av[2][8], bv[2][8];
#pragma unroll
    for (int a = 0; a < 2; ++a) {
      const f32x4v a0 = *reinterpret_cast<const f32x4v *>(arow[a] + 16 * ch);
      const f32x4v a1 = *reinterpret_cast<const f32x4v *>(arow[a] + 16 * ch + 4);
      const f32x4v b0 = *reinterpret_cast<const f32x4v *>(brow[a] + 16 * ch);
      const f32x4v b1 = *reinterpret_cast<const f32x4v *>(brow[a] + 16 * ch + 4);
#pragma unroll
      for (int i = 0; i < 4; ++i) { av[a][i] = a0[i]; av[a][4 + i] = a1[i]; bv[a][i] = b0[i]; bv[a][4 + i] = b1[i]; }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[a][i], bv[b][i], acc[a][b], 0, 0, 0);
  }
  float *out = scores + (int64_t)hb * NB * NB;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = ti * 64 + 32 * a + (r >> 2) * 8 + 4 * h + (r & 3);
        const int col = tj * 64 + 32 * b + n;
        if (row < NB && col < NB) out[(int64_t)row * NB + col] = acc[a][b][r] * scale;
      }
}

// grid (NB, heads of the batch): row b keeps its min(topk, b+1) largest logits among c <= b.
// Rows of up to 256 * BS_SEL_E logits are read once, 16 bytes per load, and held in registers
// (thread t: elements 4 t .. 4 t + 3, 1024 + 4 t .. and so on; needs NB % 4 == 0).  The k-th largest of the 256 thread maxima is a lower bound of the k-th
// largest logit (k <= 256 maxima are at least that large), so only the logits that reach it
// -- a few hundred of a long row -- go to LDS as candidates; the exact threshold is found among
// them, the kept positions are marked in two bit maps (above the threshold / equal to it) and
// written out in index order, equal logits lowest index first.  Rows that do not fit (longer
// rows, k > 256, more candidates than LDS holds, e.g. a constant row) take the general
// radix select over memory.
constexpr int BS_SEL_E = 64;
constexpr int BS_SEL_CAP = 2048;
__global__ __launch_bounds__(256) void bs_select_kernel(int NB, int slot0, int topk, const float *scores,
                                                        int32_t *blk_idx, int32_t *blk_cnt) {
  __shared__ int hist[256];
  __shared__ int sh[24];
  __shared__ unsigned ckey[BS_SEL_CAP];
  __shared__ int cidx[BS_SEL_CAP];
  __shared__ unsigned bitg[256 * BS_SEL_E / 32], bite[256 * BS_SEL_E / 32];
  const int b = blockIdx.x, hb = blockIdx.y, slot = slot0 + hb, tid = threadIdx.x;
  const float *row = scores + ((int64_t)hb * NB + b) * NB;
  int32_t *out = blk_idx + ((int64_t)slot * NB + b) * topk;
  const int n = b + 1, k = min(topk, n);
  if (tid == 0) blk_cnt[(int64_t)slot * NB + b] = k;
  if (n <= topk) {
    for (int i = tid; i < topk; i += 256) out[i] = i < n ? i : -1;
    return;
  }
  bool general = k > 256 || n > 256 * BS_SEL_E || (NB & 3) != 0;
  if (!general) {
    unsigned u[BS_SEL_E];
    unsigned mx = 0u;
#pragma unroll
    for (int j = 0; j < BS_SEL_E / 4; ++j) {
      u[4 * j] = u[4 * j + 1] = u[4 * j + 2] = u[4 * j + 3] = 0u;
      if (j * 1024 < n) {                     // wave-uniform
        const int i = j * 1024 + 4 * tid;
        if (i < n) {                          // the row's storage extends to NB >= i + 4
          const float4 a = *reinterpret_cast<const float4 *>(row + i);
          u[4 * j] = max(order_key(a.x), 1u);            // 0 marks "no element"
          if (i + 1 < n) u[4 * j + 1] = max(order_key(a.y), 1u);
          if (i + 2 < n) u[4 * j + 2] = max(order_key(a.z), 1u);
          if (i + 3 < n) u[4 * j + 3] = max(order_key(a.w), 1u);
        }
        mx = max(max(mx, u[4 * j]), max(u[4 * j + 1], max(u[4 * j + 2], u[4 * j + 3])));
      }
    }
    ckey[tid] = mx;
    __syncthreads();
    unsigned bound;
    int unused;
    radix_select_lds<256>(ckey, 256, k, &bound, &unused, hist, sh);
    bound = max(bound, 1u);
    int cnt = 0;
#pragma unroll
    for (int j = 0; j < BS_SEL_E; ++j)
      if ((j >> 2) * 1024 < n) cnt += u[j] >= bound;
    int base, e0, total, t1;
    block_scan2_256(cnt, 0, &base, &e0, &total, &t1, sh);
    general = total > BS_SEL_CAP;             // uniform over the workgroup
    if (!general) {
#pragma unroll
      for (int j = 0; j < BS_SEL_E; ++j)
        if ((j >> 2) * 1024 < n && u[j] >= bound) {
          ckey[base] = u[j];
          cidx[base] = (j >> 2) * 1024 + 4 * tid + (j & 3);
          ++base;
        }
      const int nw = (n + 31) >> 5;
      for (int w = tid; w < nw; w += 256) { bitg[w] = 0u; bite[w] = 0u; }
      __syncthreads();
      unsigned thr;
      int take_eq;
      radix_select_lds<256>(ckey, total, k, &thr, &take_eq, hist, sh);
      for (int c = tid; c < total; c += 256) {
        const unsigned key = ckey[c];
        const int i = cidx[c];
        if (key > thr) atomicOr(&bitg[i >> 5], 1u << (i & 31));
        else if (key == thr) atomicOr(&bite[i >> 5], 1u << (i & 31));
      }
      __syncthreads();
      // thread t owns the words 2t, 2t + 1 (positions 64 t .. 64 t + 63)
      unsigned G[2], E[2];
#pragma unroll
      for (int w = 0; w < 2; ++w) {
        const bool in = 2 * tid + w < nw;
        G[w] = in ? bitg[2 * tid + w] : 0u;
        E[w] = in ? bite[2 * tid + w] : 0u;
      }
      int gb, eb, tg, te;
      block_scan2_256(__builtin_popcount(G[0]) + __builtin_popcount(G[1]),
                      __builtin_popcount(E[0]) + __builtin_popcount(E[1]), &gb, &eb, &tg, &te, sh);
#pragma unroll
      for (int w = 0; w < 2; ++w) {
        unsigned m = G[w] | E[w];
        while (m) {
          const int bit = __builtin_ctz(m);
          m &= m - 1u;
          const int i = 64 * tid + 32 * w + bit;
          if ((G[w] >> bit) & 1u) {
            out[gb + min(eb, take_eq)] = i;
            ++gb;
          } else {
            if (eb < take_eq) out[gb + eb] = i;
            ++eb;
          }
        }
      }
      return;
    }
  }
  unsigned thr;
  int take_eq;
  radix_select<256, false>(row, n, k, &thr, &take_eq, hist, sh);
  ordered_select<256, false>(row, n, thr, take_eq, out, sh + 8);
}

// ---------------------------------------------------------------------------
// Block logits and per-row top-k in one kernel (Alg. 3): the NB x NB logits are never stored.
// Workgroup = 128 query blocks of one head, 16 per wave, eight waves: two per SIMD, so that one
// wave's selection work runs while the other's MFMAs occupy the matrix pipeline (a single wave
// issues in order and gets no such overlap).  Per 32-key tile (pooled K vectors staged in LDS,
// shared by the eight waves, double buffered) a wave forms its 32 x 16 logits transposed,
// S^T = K_hat Q_hat^T with the 16 x 16 x 4 fp32 MFMA, so that the four lanes n, n + 16, n + 32,
// n + 48 hold the logits of ONE query block n: the top-k state of a row is private to its four
// lanes, and no atomics or cross-row traffic are needed.
// Per row: a candidate list in LDS (order key of the logit + key block, at most BSF_CAP entries,
// in key-block order) and a bar tau: a logit enters the list iff its key exceeds tau.  When a
// list cannot take its share of a tile, its row finds by bisection a key T with at least k
// entries >= T, drops what is below, keeps of the entries equal to T only the first it still
// needs, and raises tau to T: k or more entries with a lower key block reach T, so a later logit
// <= T cannot be among the k largest (ties go to the lower block).  After the last tile the same
// step with the exact k-th largest key leaves exactly the k selected blocks, already ascending.
// Needs topk <= BSF_MAX_TOPK and NB < 65536 (block ids are kept in 16 bits).
// ---------------------------------------------------------------------------
constexpr int BSF_ROWS = 128;                       // query blocks per workgroup
constexpr int BSF_THREADS = 512;
constexpr int BSF_CAP = 160;                        // candidates a row can hold
constexpr int BSF_PITCH = 164;                      // entries between rows: a multiple of 4 (16-byte reads)
                                                    // and an odd multiple of 4 (16 rows hit 64 different banks)
constexpr int BSF_SLACK = 16;                       // the bisection of a running cut stops at k .. k + slack entries
constexpr int BSF_MAX_TOPK = BSF_CAP - 32 - BSF_SLACK;   // 32: what one tile can add to a row
constexpr int BSF_TILE_BYTES = 32 * 512;            // 32 pooled vectors of 128 floats
constexpr size_t BSF_LDS = 2 * BSF_TILE_BYTES + (size_t)BSF_ROWS * BSF_PITCH * (4 + 2);

// the lists are addressed as LDS (not through generic pointers) also inside the functions below
typedef __attribute__((address_space(3))) unsigned lds_u32;
typedef __attribute__((address_space(3))) unsigned short lds_u16;
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
typedef __attribute__((address_space(3))) u32x2 lds_u32x2;

constexpr int BSF_GROUPS = BSF_CAP / 16;            // 4-entry groups of a list that one of the row's four lanes holds

// Exchanges between the four lanes of a row (n, n + 16, n + 32, n + 48) by the lane-swap instructions
// of the vector ALU, not through the LDS crossbar, whose round trip each exchange would wait for.
// permlane16_swap(a, b) swaps the odd 16-lane rows of a with the even rows of b, permlane32_swap(a, b)
// the upper half of a with the lower half of b; with a = b = v the two results are (own, partner) in
// the lanes of an even row / the lower half and (partner, own) in the others.
__device__ __forceinline__ unsigned bsf_xor16(unsigned v) {
  const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
  return (threadIdx.x & 16) ? r[0] : r[1];
}
__device__ __forceinline__ unsigned bsf_xor32(unsigned v) {
  const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  return (threadIdx.x & 32) ? r[0] : r[1];
}
__device__ __forceinline__ int bsf_row_sum(int v) {
  const auto r = __builtin_amdgcn_permlane16_swap((unsigned)v, (unsigned)v, false, false);
  const unsigned u = r[0] + r[1];
  const auto t = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return (int)(t[0] + t[1]);
}
__device__ __forceinline__ unsigned bsf_row_max(unsigned v) {
  const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
  const unsigned u = max(r[0], r[1]);
  const auto t = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return max(t[0], t[1]);
}

// Serial form of the cut below, for a row whose entries equal to T are more than it may keep: of
// those the first `quota` in list order (the lowest key blocks) stay.  The row's first lane walks
// the list, 32 entries at a time through registers: the reads of a chunk are issued together and
// the writes land at or below positions already read.  Returns the new count (valid in that lane).
__device__ inline int bsf_cut_serial(lds_u32 *keys, lds_u16 *idx, int cnt, unsigned T, int quota, int hq) {
  int out = 0;
  if (hq == 0) {
    for (int c0 = 0; c0 < cnt; c0 += 32) {
      unsigned kv[32], bv[32];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const u32x4 e = *reinterpret_cast<const lds_u32x4 *>(keys + c0 + 4 * j);
        const u32x2 b = *reinterpret_cast<const lds_u32x2 *>(idx + c0 + 4 * j);
        kv[4 * j] = e.x; kv[4 * j + 1] = e.y; kv[4 * j + 2] = e.z; kv[4 * j + 3] = e.w;
        bv[4 * j] = b.x & 0xffffu; bv[4 * j + 1] = b.x >> 16; bv[4 * j + 2] = b.y & 0xffffu; bv[4 * j + 3] = b.y >> 16;
      }
#pragma unroll
      for (int i = 0; i < 32; ++i) {
        const unsigned v = kv[i];
        const bool live = c0 + i < cnt;                      // what lies behind the list is stale
        bool keep = v > T;
        if (v == T && quota > 0 && live) { keep = true; --quota; }
        if (keep && live) { keys[out] = v; idx[out] = (unsigned short)bv[i]; ++out; }
      }
    }
  }
  return out;
}

// Cut of one row's list (the four lanes of the row call it with the same arguments; every lane of
// the wave calls it).  tau: the row's bar, which every entry's key reaches.  A row with more than
// `limit` entries (limit = k when exact, else k + slack) finds a key T with k .. limit entries
// >= T, keeps those and raises its bar to T; the others keep what they have.  Returns the new
// count and bar.
// The lane of quarter hq holds the list's 4-entry groups hq, hq + 4, ... in registers for the
// whole step (the bisection then costs no memory access), and the four lanes write the kept
// entries back at the same time, after all reads: the position of a group is the number of kept
// entries in the groups before it, over the four lanes.  Dropped entries go to the slot behind
// the list's capacity.
// (A function of its own, not inlined: its registers would otherwise be live through the
// caller's inner loop.)
struct BsfCut { int cnt; unsigned tau; };                   // returned in registers: nothing of the caller's lives in memory
__device__ __noinline__ BsfCut bsf_compact(lds_u32 *keys, lds_u16 *idx, int cnt, int k, bool exact, int hq,
                                           unsigned tau) {
  unsigned kv[BSF_GROUPS][4];
  u32x2 bv[BSF_GROUPS];
  unsigned hi = 0u;
#pragma unroll
  for (int g = 0; g < BSF_GROUPS; ++g) {
    const int base = 16 * g + 4 * hq;                          // < BSF_CAP <= BSF_PITCH - 4: inside the row
    const u32x4 e = *reinterpret_cast<const lds_u32x4 *>(keys + base);
    bv[g] = *reinterpret_cast<const lds_u32x2 *>(idx + base);
    const unsigned v[4] = {e.x, e.y, e.z, e.w};
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      kv[g][c] = base + c < cnt ? v[c] : 0u;                   // live keys are >= 1
      hi = max(hi, kv[g][c]);
    }
  }
  hi = bsf_row_max(hi);
  auto count_ge = [&](unsigned v) {
    int c = 0;
#pragma unroll
    for (int g = 0; g < BSF_GROUPS; ++g)
#pragma unroll
      for (int j = 0; j < 4; ++j) c += kv[g][j] >= v;
    return bsf_row_sum(c);
  };
  const int limit = exact ? k : k + min(BSF_SLACK, (BSF_CAP - 32 - k) / 2);
  const bool cut = cnt > limit;
  // invariant: at least k entries are >= lo (at the start all of them: an entry exceeded the bar of
  // its time, and a cut keeps what reaches the new bar); fewer than k are > hi
  unsigned lo = tau;
  bool act = cut && lo < hi;
  while (__builtin_amdgcn_ballot_w64(act)) {
    const unsigned mid = lo + ((hi - lo + 1u) >> 1);           // lo < mid <= hi
    const int c = count_ge(mid);
    if (act) {
      if (c >= k) {
        lo = mid;
        if (c <= limit) act = false;
      } else {
        hi = mid - 1u;
      }
      if (lo >= hi) act = false;
    }
  }
  if (!cut) return BsfCut{cnt, tau};                           // nothing moves: list and bar stay
  const unsigned T = lo;
  const int reach = count_ge(T);                               // >= k
  const bool ties = reach > limit;                             // too many entries equal to T: serial cut
  int serial_cnt = 0;
  if (__builtin_amdgcn_ballot_w64(ties)) {
    if (ties) {
      const int above = T == 0xffffffffu ? 0 : count_ge(T + 1u);
      serial_cnt = bsf_cut_serial(keys, idx, cnt, T, k - above, hq);
    }
    serial_cnt = (int)bsf_row_max(hq == 0 ? (unsigned)serial_cnt : 0u);   // from the row's first lane
  }
  // kept entries per group: prefix over this lane's groups, exclusive and inclusive, one byte each
  unsigned excl[3] = {0u, 0u, 0u}, incl[3] = {0u, 0u, 0u};
  {
    int run = 0;
#pragma unroll
    for (int g = 0; g < BSF_GROUPS; ++g) {
      excl[g >> 2] |= (unsigned)run << (8 * (g & 3));
#pragma unroll
      for (int j = 0; j < 4; ++j) run += kv[g][j] >= T;
      incl[g >> 2] |= (unsigned)run << (8 * (g & 3));
    }
  }
  // list position of this lane's group g = kept entries of all groups before it: of a lane with a
  // lower quarter the groups 0 .. g, of one with a higher quarter the groups 0 .. g-1.  Each lane
  // sends each of the other three what that one needs; sums stay below 256 per byte.
  unsigned at_pk[3] = {excl[0], excl[1], excl[2]};
#pragma unroll
  for (int x = 1; x < 4; ++x) {
    const bool lower = hq < (hq ^ x);                          // this lane comes before its partner
#pragma unroll
    for (int w = 0; w < 3; ++w) {
      unsigned got = lower ? incl[w] : excl[w];
      if (x & 1) got = bsf_xor16(got);
      if (x & 2) got = bsf_xor32(got);
      at_pk[w] += got;
    }
  }
#pragma unroll
  for (int g = 0; g < BSF_GROUPS; ++g) {
    int pos = (at_pk[g >> 2] >> (8 * (g & 3))) & 255u;
    const unsigned b[4] = {bv[g].x & 0xffffu, bv[g].x >> 16, bv[g].y & 0xffffu, bv[g].y >> 16};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bool keep = kv[g][j] >= T && !ties;
      const int at = keep ? pos : BSF_CAP + hq;                // behind the capacity: slots nobody reads, one per lane
      keys[at] = kv[g][j];
      idx[at] = (unsigned short)b[j];
      pos += keep;
    }
  }
  return BsfCut{ties ? serial_cnt : reach, T};
}

// The float whose order key is the bar (below / above every real logit outside the keys of real
// floats): a logit's key exceeds the bar iff the logit exceeds this value (the two zeros count
// as equal here).
__device__ inline float bsf_bar_value(unsigned tau) {
  if (tau <= 0x007fffffu) return -__builtin_inff();
  if (tau >= 0xff800000u) return __builtin_inff();
  return __uint_as_float((tau & 0x80000000u) ? (tau & 0x7fffffffu) : ~tau);
}

// Q_hat[row][32 hq .. 32 hq + 31]: the mean of the block's 64 query rows, summed in the order of
// bs_pool_kernel (tokens r, r + 16, r + 32, r + 48 first, then r = 0 .. 15), so that both give the same bits.
__device__ __forceinline__ void bsf_pool_q(const bf16_t *q0, int64_t q_st, float (&q)[32]) {
#pragma unroll
  for (int j = 0; j < 32; ++j) q[j] = 0.f;
  for (int r = 0; r < 16; ++r) {
    float part[32];
#pragma unroll
    for (int j = 0; j < 32; ++j) part[j] = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bf16_t *p = q0 + (int64_t)(r + 16 * i) * q_st;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint4 w = *reinterpret_cast<const uint4 *>(p + 8 * c);
        const unsigned ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          part[8 * c + 2 * j] += __uint_as_float(ww[j] << 16);
          part[8 * c + 2 * j + 1] += __uint_as_float(ww[j] & 0xffff0000u);
        }
      }
    }
#pragma unroll
    for (int j = 0; j < 32; ++j) q[j] += part[j];
  }
#pragma unroll
  for (int j = 0; j < 32; ++j) q[j] *= 1.0f / 64.0f;
}

__global__ __launch_bounds__(BSF_THREADS) void bs_topk_kernel(QKV x, HeadList hl, int NB, int NBp, int topk, KvMap km,
                                                              const float *kpool, int32_t *blk_idx, int32_t *blk_cnt) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  unsigned *ckey = reinterpret_cast<unsigned *>(lds + 2 * BSF_TILE_BYTES);
  unsigned short *cidx = reinterpret_cast<unsigned short *>(ckey + BSF_ROWS * BSF_PITCH);
  const int slot = blockIdx.x;
  const int R0 = (gridDim.y - 1 - blockIdx.y) * BSF_ROWS;    // the longest rows of every head first
  const int tid = threadIdx.x, lane = tid & 63, n = lane & 15, hq = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int row = R0 + 16 * wave + n;                        // query block of these four lanes
  const bool row_ok = row < NB;
  const int k = min(topk, row + 1);
  lds_u32 *keys = (lds_u32 *)ckey + (16 * wave + n) * BSF_PITCH;    // this row's list
  lds_u16 *idx = (lds_u16 *)cidx + (16 * wave + n) * BSF_PITCH;
  int cnt = 0;
  unsigned tau = row_ok ? 0u : 0xffffffffu;                  // every entry's key reaches it; a logit enters iff its key
  float bar = bsf_bar_value(tau);                            // exceeds it.  Rows past the end take nothing.

  // B operand: Q_hat[row][32 hq + j], j = 0 .. 31 (the contraction index of the lane of quarter hq in
  // MFMA step j is 32 hq + j, for both operands), pooled here from the block's 64 query rows: the
  // pooled Q never goes through memory.
  float q[32];
  bsf_pool_q(x.q + hl.h[slot] * x.q_sh + (int64_t)(64 * min(row, NB - 1)) * x.q_st + 32 * hq, x.q_st, q);
  const float *kp = kpool + (int64_t)km.slot_kv[slot] * NBp * 128;
  const int last_row = min(R0 + BSF_ROWS, NB) - 1;           // last query block of the workgroup
  const int n_tiles = last_row / 32 + 1;                     // key tiles that hold a key <= last_row
  const int wave_first = R0 + 16 * wave;
  const int t_last = wave_first < NB ? min(wave_first + 15, NB - 1) / 32 : -1;   // last tile with a causal key for this wave

  // Tile t = pooled K rows 32 t .. 32 t + 31 (kpool is padded to whole tiles), 512 bytes each, in
  // LDS with the 16-byte chunk c of row m at chunk position c ^ (m % 16): the 16 lanes that read
  // one chunk column of 16 rows hit all 64 banks.  One load instruction fills two rows; this wave
  // issues two of the sixteen.
  auto fetch = [&](int t) {
    const float *ubase = kp + (int64_t)(32 * t) * 128;
    const unsigned base = lds_addr_of(lds + (t & 1) * BSF_TILE_BYTES);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int b = 2 * wave + i, r = 2 * b + (lane >> 5), p = lane & 31;
      const unsigned voff = (unsigned)r * 512u + (unsigned)((p ^ (r & 15)) << 4);
      dma16_su(ubase, voff, base + b * 1024);
    }
  };

  // Selection of one tile's logits sc[e], e = 4 b + r: key block kb + 16 b + 4 hq + r against this row.
  auto select = [&](const float (&sc)[8], int kb) {
    unsigned takes = 0u;
#pragma unroll
    for (int e = 0; e < 8; ++e) takes |= sc[e] > bar ? 1u << e : 0u;
    if (kb + 31 > wave_first) {                              // only a tile on the diagonal holds keys past a row
      const int rel = row - kb - 4 * hq;                     // entry e is causal iff 16 b + r <= rel
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (16 * (e >> 2) + (e & 3) > rel) takes &= ~(1u << e);
    }
    if (__builtin_amdgcn_ballot_w64(takes != 0u) == 0) return;
    // A list that cannot take its share of this tile: every row of the wave that holds more than
    // it must is cut down with it (the rows then fill up together: one cut where the wave would
    // pay for sixteen), and what the raised bars exclude leaves the tile's share.  A cut leaves a
    // row at most BSF_CAP - 32 entries, so its share fits.
    // (counts of the tile's two 16-key blocks, one byte each, from all four lanes: of the lanes hq ^ 1, hq ^ 2, hq ^ 3)
    unsigned mine = (unsigned)__builtin_popcount(takes & 15u) | (unsigned)__builtin_popcount(takes >> 4) << 8;
    unsigned p1 = bsf_xor16(mine), p2 = bsf_xor32(mine), p3 = bsf_xor32(p1);
    unsigned all = mine + p1 + p2 + p3;
    if (__builtin_amdgcn_ballot_w64(cnt + (int)(all & 255u) + (int)(all >> 8) > BSF_CAP)) {
      const BsfCut c = bsf_compact(keys, idx, cnt, k, false, hq, tau);
      cnt = c.cnt; tau = c.tau;
      bar = bsf_bar_value(tau);
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (!(sc[e] > bar)) takes &= ~(1u << e);
      mine = (unsigned)__builtin_popcount(takes & 15u) | (unsigned)__builtin_popcount(takes >> 4) << 8;
      p1 = bsf_xor16(mine); p2 = bsf_xor32(mine); p3 = bsf_xor32(p1);
      all = mine + p1 + p2 + p3;
    }
    // list order = key-block order: within a 16-key block the four lanes of the row follow each
    // other with four keys each
    const unsigned before = ((hq ^ 1) < hq ? p1 : 0u) + ((hq ^ 2) < hq ? p2 : 0u) + ((hq ^ 3) < hq ? p3 : 0u);
    int pos = cnt + (int)(before & 255u);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if (e == 4) pos = cnt + (int)(all & 255u) + (int)(before >> 8);
      const bool take = (takes >> e) & 1u;
      const int at = take ? pos : BSF_CAP + hq;              // an entry that does not enter goes behind the list (a slot per lane)
      keys[at] = max(order_key(sc[e]), 1u);
      idx[at] = (unsigned short)(kb + 16 * (e >> 2) + 4 * hq + (e & 3));
      pos += take;
    }
    cnt += (int)(all & 255u) + (int)(all >> 8);
  };

  fetch(0);
  for (int t = 0; t < n_tiles; ++t) {
    __builtin_amdgcn_s_waitcnt(0x0F70);                      // vmcnt(0), as an instruction the compiler's own wait counting sees
    __syncthreads();                                         // tile t landed; every wave is done with tile t-1
    if (t + 1 < n_tiles) fetch(t + 1);
    if (t > t_last) continue;                                // no key of the tile is causal for this wave
    const int kb = 32 * t;
    // logits of the tile's two 16-key blocks, two accumulation chains each
    const char *tile = lds + (t & 1) * BSF_TILE_BYTES + n * 512;
    f32x4v acc[2][2];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int c = 0; c < 2; ++c) acc[b][c] = f32x4v{0.f, 0.f, 0.f, 0.f};
    float4 a0[8], a1[8];                                     // all of the tile's operands first: one LDS latency, not eight
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int ch = ((8 * hq + i) ^ n) << 4;                // rows n and 16 + n share n % 16
      a0[i] = *reinterpret_cast<const float4 *>(tile + ch);
      a1[i] = *reinterpret_cast<const float4 *>(tile + 16 * 512 + ch);
    }
    __builtin_amdgcn_sched_barrier(0);                       // keeps the loads up here, ahead of the MFMAs
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      acc[0][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0[i].x, q[4 * i], acc[0][0], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1[i].x, q[4 * i], acc[1][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0[i].y, q[4 * i + 1], acc[0][1], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1[i].y, q[4 * i + 1], acc[1][1], 0, 0, 0);
      acc[0][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0[i].z, q[4 * i + 2], acc[0][0], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1[i].z, q[4 * i + 2], acc[1][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0[i].w, q[4 * i + 3], acc[0][1], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1[i].w, q[4 * i + 3], acc[1][1], 0, 0, 0);
    }
    float sc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) sc[e] = acc[e >> 2][0][e & 3] + acc[e >> 2][1][e & 3];
    select(sc, kb);
  }
  // exact selection of what is left, then the row goes out (ascending; -1 behind the last entry)
  cnt = bsf_compact(keys, idx, cnt, k, true, hq, tau).cnt;
  if (row_ok) {
    int32_t *out = blk_idx + ((int64_t)slot * NB + row) * topk;
    for (int i = hq; i < topk; i += 4) out[i] = i < cnt ? (int32_t)idx[i] : -1;
    if (hq == 0) blk_cnt[(int64_t)slot * NB + row] = cnt;
  }
}

// Processing order of the query blocks of one head: sorted by (first kept key block, block id).
// One workgroup per head: the composite keys (first << 16 | block) of up to 32768 blocks are
// sorted in LDS (4 bytes per block, up to 128 KiB) by a bitonic network (padded to a power of
// two with keys above every real one).
constexpr int BS_ORDER_MAX = 32768;
__global__ __launch_bounds__(1024) void bs_order_kernel(int NB, int topk, const int32_t *blk_idx, int32_t *order) {
  extern __shared__ unsigned key[];
  const int slot = blockIdx.x, tid = threadIdx.x;
  const int32_t *idx = blk_idx + (int64_t)slot * NB * topk;
  int32_t *out = order + (int64_t)slot * NB;
  int P = 1024;
  while (P < NB) P <<= 1;
  for (int b = tid; b < P; b += 1024) {
    unsigned kf = 0xffffu;
    if (b < NB) {
      const int f = idx[(int64_t)b * topk];
      kf = f < 0 ? 0u : (f > 0xfffe ? 0xfffeu : (unsigned)f);
    }
    key[b] = (kf << 16) | (unsigned)(b & 0xffff);
  }
  __syncthreads();
  for (int k = 2; k <= P; k <<= 1)
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int i = tid; i < P; i += 1024) {
        const int l = i ^ j;
        if (l > i) {
          const unsigned a = key[i], c = key[l];
          const bool up = (i & k) == 0;
          if ((a > c) == up) { key[i] = c; key[l] = a; }
        }
      }
      __syncthreads();
    }
  for (int b = tid; b < NB; b += 1024) out[b] = (int32_t)(key[b] & 0xffffu);
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
static inline size_t align256(size_t v) { return (v + 255) / 256 * 256; }

static int vs_chunk_keys(int N) { return N <= VS_TINY_N ? VS_CHUNK_TINY : N <= VS_SHORT_N ? VS_CHUNK_SHORT : VS_CHUNK; }
static int vs_chunks(int N) { return (N + vs_chunk_keys(N) - 1) / vs_chunk_keys(N); }

static int vs_slices(int N) { return (N + VS_SLICE - 1) / VS_SLICE; }
static int vs_cand_cap(int N) { return N / 4 > 1024 ? N / 4 : 1024; }        // candidates per (head, which)

size_t vs_index_ws_bytes(int N, int n_heads) {
  size_t b = 0;
  b += 2 * align256((size_t)n_heads * N * sizeof(float));                     // colsum, diagsum
  b += align256((size_t)n_heads * vs_chunks(N) * 128 * sizeof(float));        // per-chunk (max, sum)
  b += align256((size_t)n_heads * 128 * sizeof(float));                       // final (max, 1/sum)
  b += 2 * align256((size_t)n_heads * (N / 4) * sizeof(float));               // group maxima (G >= 4)
  b += 4 * align256((size_t)n_heads * 2 * vs_cand_cap(N) * sizeof(float));    // candidates: parts and list, value and position
  b += align256((size_t)n_heads * 2 * vs_slices(N) * sizeof(int2));           // where every slice put its part
  b += align256((size_t)n_heads * 2 * sizeof(VsSelState));
  return b;
}

hipError_t launch_build_vs(const QKV &x, const HeadList &hl, int last_q, int nv, int ns,
                           int32_t *v_idx, int32_t *s_idx, int32_t *cover, uint32_t *cover_bits,
                           int32_t *counts, int cover_words, void *ws, hipStream_t st) {
  const int N = x.N, nc = vs_chunks(N);
  char *p = static_cast<char *>(ws);
  float *colsum = reinterpret_cast<float *>(p); p += align256((size_t)hl.n * N * sizeof(float));
  float *diagsum = reinterpret_cast<float *>(p); p += align256((size_t)hl.n * N * sizeof(float));
  float *ml_part = reinterpret_cast<float *>(p); p += align256((size_t)hl.n * nc * 128 * sizeof(float));
  float *ml_fin = reinterpret_cast<float *>(p); p += align256((size_t)hl.n * 128 * sizeof(float));
  const int cap = vs_cand_cap(N), n_slices = vs_slices(N);
  float *gmax_v = reinterpret_cast<float *>(p); p += align256((size_t)hl.n * (N / 4) * sizeof(float));
  float *gmax_s = reinterpret_cast<float *>(p); p += align256((size_t)hl.n * (N / 4) * sizeof(float));
  const size_t cand_bytes = align256((size_t)hl.n * 2 * cap * sizeof(float));
  float *cand_val = reinterpret_cast<float *>(p); p += cand_bytes;
  int32_t *cand_idx = reinterpret_cast<int32_t *>(p); p += cand_bytes;
  float *list_val = reinterpret_cast<float *>(p); p += cand_bytes;
  int32_t *list_idx = reinterpret_cast<int32_t *>(p); p += cand_bytes;
  int2 *seg = reinterpret_cast<int2 *>(p); p += align256((size_t)hl.n * 2 * n_slices * sizeof(int2));
  VsSelState *state = reinterpret_cast<VsSelState *>(p);
  // the listed heads grouped by K/V head, in order of first appearance, at most four per group
  VsGroups vg;
  memset(&vg, 0, sizeof(vg));
  int gkv[MINF_MAX_HEADS];
  for (int i = 0; i < hl.n; ++i) {
    const int kv = hl.h[i] / x.group;
    int g = 0;
    while (g < vg.n && !(gkv[g] == kv && vg.cnt[g] < VS_GROUP)) ++g;
    if (g == vg.n) { gkv[g] = kv; ++vg.n; }
    vg.slot[g][vg.cnt[g]++] = (uint8_t)i;
  }
  // 48 KiB (three workgroups of four waves per CU; registers allow two) and 75 KiB (two per CU)
  const dim3 grid(nc, vg.n);
  auto score = [&](auto chunk_keys) -> hipError_t {
    constexpr int C = decltype(chunk_keys)::value;
    const size_t lds1 = 3 * VS_TILE_BYTES;
    const size_t lds2 = 3 * HALF_BYTES + VS_GROUP * vs_wave_floats(C) * sizeof(float);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(vs_score_kernel<2, C>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds2);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((vs_score_kernel<1, C>), grid, dim3(256), lds1, st, x, hl, vg, last_q, nc, ml_part,
                       (const float *)nullptr, (float *)nullptr, (float *)nullptr);
    hipLaunchKernelGGL(vs_combine_kernel, dim3(hl.n), dim3(1024), 0, st, nc, (const float *)ml_part, ml_fin);
    hipLaunchKernelGGL((vs_score_kernel<2, C>), grid, dim3(256), lds2, st, x, hl, vg, last_q, nc, (float *)nullptr,
                       (const float *)ml_fin, colsum, diagsum);
    return hipSuccess;
  };
  const int ck = vs_chunk_keys(N);
  const hipError_t e = ck == VS_CHUNK_TINY    ? score(std::integral_constant<int, VS_CHUNK_TINY>{})
                       : ck == VS_CHUNK_SHORT ? score(std::integral_constant<int, VS_CHUNK_SHORT>{})
                                              : score(std::integral_constant<int, VS_CHUNK>{});
  if (e != hipSuccess) return e;
  // top-k of the line scores: prefilter by many workgroups, exact selection on what is left
  const int kv_ = nv < N ? nv : N, ks_ = ns < N ? ns : N;
  const int log_gv = vs_log_group(N, kv_), log_gs = vs_log_group(N, ks_);
  if (log_gv >= 0 || log_gs >= 0)
    hipLaunchKernelGGL(vs_gmax_kernel, dim3((N + 4095) / 4096, hl.n, 2), dim3(256), 0, st, N, log_gv, log_gs,
                       (const float *)colsum, (const float *)diagsum, gmax_v, gmax_s);
  const bool prefilter = log_gv >= 0 || log_gs >= 0;
  if (prefilter)
    hipLaunchKernelGGL(vs_bound_kernel, dim3(hl.n, 2), dim3(1024), 0, st, N, nv, ns, log_gv, log_gs,
                       (const float *)gmax_v, (const float *)gmax_s, state);
  if (prefilter)
    hipLaunchKernelGGL(vs_filter_kernel, dim3(n_slices, hl.n, 2), dim3(256), 0, st, N, cap, n_slices,
                       (const float *)colsum, (const float *)diagsum, state, cand_val, cand_idx, seg);
  hipLaunchKernelGGL(vs_select_kernel, dim3(hl.n, 2), dim3(1024), 0, st, N, nv, ns, (const float *)colsum,
                     (const float *)diagsum, v_idx, s_idx, cover, cover_bits, counts, cover_words, cap,
                     prefilter ? n_slices : 0, (const VsSelState *)state, (const float *)cand_val, (const int32_t *)cand_idx,
                     (const int2 *)seg, list_val, list_idx);
  return hipGetLastError();
}

hipError_t launch_vs_lines(int N, int rows, int nv, int ns, const int32_t *s_idx, int32_t *cover,
                           uint32_t *cover_bits, int32_t *counts, int cover_words, hipStream_t st) {
  hipLaunchKernelGGL(vs_lines_kernel, dim3(rows), dim3(1024), 0, st, N, nv, ns, s_idx, cover, cover_bits, counts,
                     cover_words);
  return hipGetLastError();
}

// Block logits are staged in the workspace for at most this many bytes at a
// time; heads are processed in batches that fit.
static const size_t BS_SCORE_CAP = (size_t)2 << 30;

static int bs_head_batch(int NB, int n_heads) {
  const size_t per = (size_t)NB * NB * sizeof(float);
  size_t hb = BS_SCORE_CAP / per;
  if (hb < 1) hb = 1;
  return (int)(hb < (size_t)n_heads ? hb : (size_t)n_heads);
}

static int bs_rows_padded(int NB) { return (NB + 31) / 32 * 32; }
static bool bs_fused(int NB, int topk) { return topk <= BSF_MAX_TOPK && NB < 65536; }

size_t bs_index_ws_bytes(int N, int n_heads, int topk) {
  const int NB = N / 64;
  size_t b = 0;
  b += align256((size_t)n_heads * bs_rows_padded(NB) * 128 * sizeof(float));   // pooled K, whole 32-row tiles
  if (!bs_fused(NB, topk)) {
    b += align256((size_t)n_heads * NB * 128 * sizeof(float));                 // pooled Q
    b += align256((size_t)bs_head_batch(NB, n_heads) * NB * NB * sizeof(float)); // block logits
  }
  return b;
}

static __global__ void iota_kernel(int n, int period, int32_t *out) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = i % period;
}

hipError_t launch_build_bs(const QKV &x, const HeadList &hl, int topk, int32_t *blk_idx,
                           int32_t *blk_cnt, int32_t *order, void *ws, hipStream_t st) {
  const int NB = x.N / 64;
  KvMap km;
  km.n_kv = 0;
  for (int i = 0; i < hl.n; ++i) {
    const int kv = hl.h[i] / x.group;
    int j = 0;
    while (j < km.n_kv && km.kv[j] != kv) ++j;
    if (j == km.n_kv) km.kv[km.n_kv++] = kv;
    km.slot_kv[i] = j;
  }
  for (int i = hl.n; i < MINF_MAX_HEADS; ++i) km.slot_kv[i] = 0;
  for (int i = km.n_kv; i < MINF_MAX_HEADS; ++i) km.kv[i] = 0;
  const int NBp = bs_rows_padded(NB);
  char *p = static_cast<char *>(ws);
  const bool fused = bs_fused(NB, topk);
  float *kpool = reinterpret_cast<float *>(p); p += align256((size_t)hl.n * NBp * 128 * sizeof(float));
  float *qpool = nullptr;
  if (!fused) { qpool = reinterpret_cast<float *>(p); p += align256((size_t)hl.n * NB * 128 * sizeof(float)); }
  float *scores = reinterpret_cast<float *>(p);
  hipLaunchKernelGGL(bs_pool_kernel, dim3(NB, (fused ? 0 : hl.n) + km.n_kv), dim3(256), 0, st, x, hl, km, qpool, kpool,
                     NBp);
  if (fused) {
    // pooling of Q, block logits and top-k in one kernel: neither the pooled Q nor anything of size NB x NB is stored
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(bs_topk_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)BSF_LDS);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(bs_topk_kernel, dim3(hl.n, (NB + BSF_ROWS - 1) / BSF_ROWS), dim3(BSF_THREADS), BSF_LDS, st, x, hl,
                       NB, NBp, topk, km, (const float *)kpool, blk_idx, blk_cnt);
  } else {
    // budgets beyond the candidate lists of the fused kernel: logits through memory, head batches
    const int hbmax = bs_head_batch(NB, hl.n);
    const int TB = (NB + 63) / 64, n_tiles = TB * (TB + 1) / 2;
    for (int s0 = 0; s0 < hl.n; s0 += hbmax) {
      const int hb = hl.n - s0 < hbmax ? hl.n - s0 : hbmax;
      hipLaunchKernelGGL(bs_logits_kernel, dim3(n_tiles, hb), dim3(64), 0, st, NB, NBp, s0, km,
                         (const float *)qpool, (const float *)kpool, scores, x.scale);
      hipLaunchKernelGGL(bs_select_kernel, dim3(NB, hb), dim3(256), 0, st, NB, s0, topk,
                         (const float *)scores, blk_idx, blk_cnt);
    }
  }
  if (order) {
    if (NB <= BS_ORDER_MAX) {
      int P = 1024;
      while (P < NB) P <<= 1;
      const size_t lds = (size_t)P * sizeof(unsigned);
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(bs_order_kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return e;
      hipLaunchKernelGGL(bs_order_kernel, dim3(hl.n), dim3(1024), lds, st, NB, topk, (const int32_t *)blk_idx, order);
    }
    else      // longer than the sort holds: natural order
      hipLaunchKernelGGL(iota_kernel, dim3((hl.n * NB + 255) / 256), dim3(256), 0, st, hl.n * NB, NB, order);
  }
  return hipGetLastError();
}

}  // namespace minf
