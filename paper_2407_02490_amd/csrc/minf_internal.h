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

// Mapping of hardware workgroup ids to logical work items.  Consecutive
// hardware ids land on different XCDs (8 of them, each with its own L2), so a
// logical id is formed as (id % 8) * per_xcd + id / 8: every XCD then walks a
// contiguous range of logical items and neighbours share K/V in its L2.
struct Sched {
  int32_t total, per_xcd;
};
inline Sched make_sched(int64_t total) {
  Sched s;
  s.total = (int32_t)total;
  s.per_xcd = (int32_t)((total + 7) / 8);
  return s;
}
__device__ inline int logical_wg(const Sched &s) {
  int hw = blockIdx.x;
  int l = (hw & 7) * s.per_xcd + (hw >> 3);
  return l < s.total ? l : -1;
}

// attention launches (attn_kernels.hip)
hipError_t launch_ashape(const QKV &x, const HeadList &hl, int n_init, int n_local, hipStream_t st);
hipError_t launch_bs(const QKV &x, const HeadList &hl, const int32_t *blk_idx, const int32_t *blk_cnt,
                     int topk, hipStream_t st);
hipError_t launch_vs(const QKV &x, const HeadList &hl, const int32_t *v_idx, const int32_t *cover,
                     const uint32_t *cover_bits, const int32_t *counts, int nv, int ns,
                     int cover_words, hipStream_t st);

// index launches (index_kernels.hip)
size_t vs_index_ws_bytes(int N, int n_heads);
size_t bs_index_ws_bytes(int N, int n_heads);
hipError_t launch_build_vs(const QKV &x, const HeadList &hl, int last_q, int nv, int ns,
                           int32_t *v_idx, int32_t *s_idx, int32_t *cover, uint32_t *cover_bits,
                           int32_t *counts, int cover_words, void *ws, hipStream_t st);
hipError_t launch_build_bs(const QKV &x, const HeadList &hl, int topk, int32_t *blk_idx,
                           int32_t *blk_cnt, void *ws, hipStream_t st);

}  // namespace minf
#endif
