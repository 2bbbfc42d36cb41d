// Internal declarations shared by the HIP translation units of libminf.
// Nothing here is part of the C ABI (see include/minf.h).
#ifndef MINF_INTERNAL_H_
#define MINF_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "minf.h"

namespace minf {

typedef __bf16 bf16_t;

// Per-call view of Q/K/V/O for one batch element (device pointers, strides in
// elements).  c_log2 = softmax_scale * log2(e): logits are scaled into the
// base-2 domain so that exp is a bare v_exp_f32.
struct QKV {
  const bf16_t *q, *k, *v;
  bf16_t *o;
  int64_t q_sh, q_st, k_sh, k_st, v_sh, v_st, o_sh, o_st;
  int32_t N, group;
  float scale, c_log2;
};

// Head ids of one call, passed to kernels by value.
struct HeadList {
  int32_t n;
  int32_t h[MINF_MAX_HEADS];
};

// Mapping of hardware workgroup ids to work items (head slot, block).
// Consecutive hardware ids land on different XCDs (8 of them, each with its own
// 4 MB L2), and workgroups are handed to the XCDs in order, so an XCD whose
// workgroups run longer than the others' starves the rest of the chip
// (measured: per-XCD head ranges cost 44% idle time on heads of unequal
// weight).  Therefore every XCD gets the same mix at every moment: heads are
// taken in chunks; inside a chunk the blocks, heaviest (last) first, are cut
// into stripes of `stripe` consecutive blocks that are dealt to the XCDs in
// serpentine order; inside a stripe the order is (block, head).  A chunk is a
// run of consecutive list slots whose heads read the same K/V head (at most 8):
// the workgroups resident on one XCD at a time are then a few neighbouring blocks
// of one GQA group and share their K/V tiles in that XCD's L2, all XCDs work on
// the same K/V head at once, and the K/V heads in flight stay few enough for the
// memory-side cache (measured at 1M tokens: chunks that mix K/V heads cost 6% on
// Vertical-Slash and 11% on Block-Sparse attention).
struct Sched {
  int32_t n_heads, n_blk, stripe, ls;   // ls = stripes per XCD per chunk
  int32_t per_xcd;                      // workgroups per XCD (grid = 8 * per_xcd)
  uint8_t cstart[MINF_MAX_HEADS];       // per list slot: first slot of its chunk
  uint8_t csize[MINF_MAX_HEADS];        // per list slot: size of its chunk
};
constexpr int SCHED_MAX_CHUNK = 8;
inline Sched make_sched(const HeadList &hl, int group, int n_blk) {
  Sched s;
  s.n_heads = hl.n;
  s.n_blk = n_blk;
  int stripe = n_blk / 64;
  s.stripe = stripe < 1 ? 1 : (stripe > 32 ? 32 : stripe);
  const int n_stripes = (n_blk + s.stripe - 1) / s.stripe;
  s.ls = (n_stripes + 7) / 8;
  s.per_xcd = s.ls * s.stripe * hl.n;      // sum over chunks of ls * stripe * chunk size
  for (int i = 0; i < MINF_MAX_HEADS; ++i) s.cstart[i] = s.csize[i] = 0;
  for (int i = 0; i < hl.n;) {
    int j = i + 1;
    while (j < hl.n && j - i < SCHED_MAX_CHUNK && hl.h[j] / group == hl.h[i] / group) ++j;
    for (int t = i; t < j; ++t) {
      s.cstart[t] = (uint8_t)i;
      s.csize[t] = (uint8_t)(j - i);
    }
    i = j;
  }
  return s;
}
// Work item of position hw (0 <= hw < 8 * per_xcd) of the launch order; false if that position
// holds none.  Plain integer arithmetic: also compiled for the host, where a test enumerates it.
__host__ __device__ inline bool decode_item(const Sched &s, int hw, int &slot, int &blk) {
  const int xcd = hw & 7;
  int seq = hw >> 3;
  // every head contributes ls * stripe items per XCD, so the chunk follows from the head position
  const int per_head = s.ls * s.stripe;
  const int hpos = seq / per_head;
  const int c0 = s.cstart[hpos], csize = s.csize[hpos];
  seq -= c0 * per_head;
  const int per_stripe = s.stripe * csize;
  const int lstripe = seq / per_stripe;
  const int r = seq - lstripe * per_stripe;
  // stripes are dealt to the XCDs in serpentine order (0..7, 7..0, ...) so that work that
  // grows with the block index (dense causal) stays balanced across XCDs
  const int pos = (lstripe & 1) ? 7 - xcd : xcd;
  const int rank = (lstripe * 8 + pos) * s.stripe + r / csize;   // 0 = last block
  slot = c0 + r % csize;
  blk = s.n_blk - 1 - rank;
  return rank < s.n_blk;
}
// Two launches in one (Vertical-Slash and Block-Sparse heads of a layer): workgroup ids come in groups of
// 40 = 32 positions of the first launch order and 8 of the second, so that the two kinds are interleaved
// four to one and a position's low three bits stay the XCD of the hardware id.  kind 0: first, 1: second.
// Returns false if the id holds no item.  groups = max(ceil(8 a.per_xcd / 32), b.per_xcd), grid = 40 groups.
__host__ __device__ inline int mixed_groups(const Sched &a, const Sched &b) {
  const int ga = (8 * a.per_xcd + 31) / 32;
  return ga > b.per_xcd ? ga : b.per_xcd;
}
__host__ __device__ inline bool decode_mixed(const Sched &a, const Sched &b, int w, int &kind, int &slot, int &blk) {
  const int g = w / 40, r = w - 40 * g, xcd = r & 7, q = r >> 3;
  kind = q < 4 ? 0 : 1;
  const Sched &s = kind == 0 ? a : b;
  const int hw = kind == 0 ? (4 * g + q) * 8 + xcd : g * 8 + xcd;
  return hw < 8 * s.per_xcd && decode_item(s, hw, slot, blk);
}
// Returns false if this workgroup has no work item.
__device__ inline bool decode_wg(const Sched &s, int &slot, int &blk) {
  return decode_item(s, blockIdx.x, slot, blk);
}

// attention launches (attn_kernels.hip)
hipError_t launch_ashape(const QKV &x, const HeadList &hl, int n_init, int n_local, hipStream_t st);
hipError_t launch_bs(const QKV &x, const HeadList &hl, const int32_t *blk_idx, const int32_t *blk_cnt,
                     const int32_t *order, int topk, hipStream_t st);
hipError_t launch_vs(const QKV &x, const HeadList &hl, const int32_t *v_idx, const int32_t *cover,
                     const uint32_t *cover_bits, const int32_t *counts, int nv, int ns,
                     int cover_words, hipStream_t st);

hipError_t launch_vs_bs(const QKV &x, const HeadList &hv, const int32_t *v_idx, const int32_t *cover,
                        const uint32_t *cover_bits, const int32_t *counts, int nv, int ns, int cover_words,
                        const HeadList &hb, const int32_t *blk_idx, const int32_t *blk_cnt, const int32_t *order,
                        int topk, hipStream_t st);

// index launches (index_kernels.hip)
size_t vs_index_ws_bytes(int N, int n_heads);
size_t bs_index_ws_bytes(int N, int n_heads, int topk);
hipError_t launch_build_vs(const QKV &x, const HeadList &hl, int last_q, int nv, int ns,
                           int32_t *v_idx, int32_t *s_idx, int32_t *cover, uint32_t *cover_bits,
                           int32_t *counts, int cover_words, void *ws, hipStream_t st);
hipError_t launch_vs_lines(int N, int rows, int nv, int ns, const int32_t *s_idx, int32_t *cover,
                           uint32_t *cover_bits, int32_t *counts, int cover_words, hipStream_t st);
hipError_t launch_build_bs(const QKV &x, const HeadList &hl, int topk, int32_t *blk_idx,
                           int32_t *blk_cnt, int32_t *order, void *ws, hipStream_t st);

}  // namespace minf
#endif
