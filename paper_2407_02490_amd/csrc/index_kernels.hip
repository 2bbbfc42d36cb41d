// placeholder, replaced below
#include "minf_internal.h"
namespace minf {
size_t vs_index_ws_bytes(int N, int n_heads) { return 256; }
size_t bs_index_ws_bytes(int N, int n_heads) { return 256; }
hipError_t launch_build_vs(const QKV &x, const HeadList &hl, int last_q, int nv, int ns,
                           int32_t *v_idx, int32_t *s_idx, int32_t *cover, uint32_t *cover_bits,
                           int32_t *counts, int cover_words, void *ws, hipStream_t st) { return hipErrorNotSupported; }
hipError_t launch_build_bs(const QKV &x, const HeadList &hl, int topk, int32_t *blk_idx,
                           int32_t *blk_cnt, void *ws, hipStream_t st) { return hipErrorNotSupported; }
}
