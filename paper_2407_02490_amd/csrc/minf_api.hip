// C ABI of libminf: argument validation and kernel launches.  Every entry
// point validates on the host first; nothing is enqueued unless all checks
// pass.  No allocation, no synchronisation.
#include <math.h>
#include <string.h>

#include <mutex>

#include "minf_internal.h"

using namespace minf;

// Scratch memory of minf_build_vs_index_noalloc: line scores and partial softmax statistics of
// the Vertical-Slash index build.  One copy per GPU, held until the process ends.  In host code
// the array's name is only a handle for hipGetSymbolAddress; the device address it yields (one
// per device) is what the kernels receive.  (No `used` attribute: the compiler gives a static
// device variable that host code names a visible symbol in the code object, which the runtime's
// lookup needs, only without it.)
static __device__ __align__(256) unsigned char scratch[MINF_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
void *g_scratch_ptr[MAX_DEVICES];          // device address of `scratch` on each device, once looked up
std::mutex g_scratch_mutex;

// Device address of the scratch array on the current device (looked up on the first call on
// that device, with that device current).  nullptr if the runtime refuses.
void *scratch_on_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}

minf_status check_qkv(const minf_qkv *x, bool need_v_o) {
  if (!x || !x->q || !x->k) return MINF_ERR_NULL;
  if (need_v_o && (!x->v || !x->o)) return MINF_ERR_NULL;
  if (x->head_dim != 128) return MINF_ERR_SHAPE;
  if (x->seq_len < MINF_BLOCK || x->seq_len % MINF_BLOCK != 0) return MINF_ERR_SHAPE;
  if (x->batch < 1 || x->n_q_heads < 1 || x->n_kv_heads < 1) return MINF_ERR_SHAPE;
  if (x->n_q_heads % x->n_kv_heads != 0) return MINF_ERR_SHAPE;
  if (!(x->softmax_scale >= 0.f) || isinf(x->softmax_scale)) return MINF_ERR_SHAPE;
  // rows are read with 16-byte accesses: token and head strides must keep that alignment
  const int64_t *s[4] = {x->q_stride, x->k_stride, x->v_stride, x->o_stride};
  for (int t = 0; t < 4; ++t) {
    if (!need_v_o && t >= 2) break;
    for (int i = 0; i < 3; ++i)
      if (s[t][i] < 0 || s[t][i] % 8 != 0) return MINF_ERR_SHAPE;
    if (s[t][2] < x->head_dim) return MINF_ERR_SHAPE;
    if (s[t][2] > (int64_t)1 << 24) return MINF_ERR_SHAPE;   // 64 rows * stride * 2 B must fit 32 bits
  }
  const void *p[4] = {x->q, x->k, x->v, x->o};
  for (int t = 0; t < (need_v_o ? 4 : 2); ++t)
    if (reinterpret_cast<uintptr_t>(p[t]) % 16 != 0) return MINF_ERR_SHAPE;
  return MINF_OK;
}

minf_status check_heads(const minf_qkv *x, const int32_t *heads, int32_t n_heads, HeadList &hl) {
  if (!heads) return MINF_ERR_NULL;
  if (n_heads < 1 || n_heads > MINF_MAX_HEADS) return MINF_ERR_SHAPE;
  memset(&hl, 0, sizeof(hl));
  hl.n = n_heads;
  for (int i = 0; i < n_heads; ++i) {
    if (heads[i] < 0 || heads[i] >= x->n_q_heads) return MINF_ERR_SHAPE;
    hl.h[i] = heads[i];
  }
  return MINF_OK;
}

QKV view(const minf_qkv *x, int b) {
  QKV v;
  v.q = static_cast<const bf16_t *>(x->q) + b * x->q_stride[0];
  v.k = static_cast<const bf16_t *>(x->k) + b * x->k_stride[0];
  v.v = x->v ? static_cast<const bf16_t *>(x->v) + b * x->v_stride[0] : nullptr;
  v.o = x->o ? static_cast<bf16_t *>(x->o) + b * x->o_stride[0] : nullptr;
  v.q_sh = x->q_stride[1]; v.q_st = x->q_stride[2];
  v.k_sh = x->k_stride[1]; v.k_st = x->k_stride[2];
  v.v_sh = x->v_stride[1]; v.v_st = x->v_stride[2];
  v.o_sh = x->o_stride[1]; v.o_st = x->o_stride[2];
  v.N = x->seq_len;
  v.group = x->n_q_heads / x->n_kv_heads;
  v.scale = x->softmax_scale > 0.f ? x->softmax_scale : 1.0f / sqrtf((float)x->head_dim);
  v.c_log2 = v.scale * 1.4426950408889634f;
  return v;
}

inline minf_status from_hip(hipError_t e) { return e == hipSuccess ? MINF_OK : MINF_ERR_HIP; }

}  // namespace

extern "C" {

const char *minf_status_string(minf_status s) {
  switch (s) {
    case MINF_OK: return "ok";
    case MINF_ERR_NULL: return "null pointer";
    case MINF_ERR_SHAPE: return "unsupported shape, stride, alignment or head list";
    case MINF_ERR_BUDGET: return "budget out of range";
    case MINF_ERR_WORKSPACE: return "workspace missing or too small";
    case MINF_ERR_UNSUPPORTED: return "unsupported parameter";
    case MINF_ERR_HIP: return "HIP launch failed";
  }
  return "unknown status";
}

int32_t minf_vs_cover_words(int32_t seq_len) {
  if (seq_len < 1) return 0;
  return (seq_len + MINF_BLOCK + 31) / 32 + 1;
}

size_t minf_vs_index_workspace_bytes(const minf_qkv *x, int32_t n_heads, int32_t last_q) {
  if (check_qkv(x, false) != MINF_OK || n_heads < 1 || n_heads > MINF_MAX_HEADS) return 0;
  if (last_q < 1 || last_q > 64) return 0;
  return vs_index_ws_bytes(x->seq_len, n_heads);
}

size_t minf_bs_index_workspace_bytes(const minf_qkv *x, int32_t n_heads, int32_t topk) {
  if (check_qkv(x, false) != MINF_OK || n_heads < 1 || n_heads > MINF_MAX_HEADS || topk < 1) return 0;
  return bs_index_ws_bytes(x->seq_len, n_heads, topk);
}

static minf_status build_vs_common(const minf_qkv *x, const int32_t *heads, int32_t n_heads, int32_t last_q,
                                   int32_t nv, int32_t ns, int32_t block, minf_vs_index *out, void *ws,
                                   size_t ws_bytes, bool own_scratch, void *hip_stream) {
  minf_status s = check_qkv(x, false);
  if (s != MINF_OK) return s;
  HeadList hl;
  if ((s = check_heads(x, heads, n_heads, hl)) != MINF_OK) return s;
  if (block != MINF_BLOCK) return MINF_ERR_UNSUPPORTED;
  if (last_q < 1 || last_q > 64 || nv < 1 || ns < 1) return MINF_ERR_BUDGET;
  if (!out || !out->v_idx || !out->s_idx || !out->cover || !out->cover_bits || !out->counts)
    return MINF_ERR_NULL;
  if (out->nv != nv || out->ns != ns || out->block != block) return MINF_ERR_BUDGET;
  if (out->cover_words < minf_vs_cover_words(x->seq_len)) return MINF_ERR_SHAPE;
  const size_t need = vs_index_ws_bytes(x->seq_len, n_heads);
  if (own_scratch) {
    if (need > (size_t)MINF_NOALLOC_SCRATCH_BYTES) return MINF_ERR_WORKSPACE;
    ws = scratch_on_current_device();
    if (!ws) return MINF_ERR_HIP;
  } else {
    if (!ws || ws_bytes < need) return MINF_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) return MINF_ERR_WORKSPACE;
  }
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  for (int b = 0; b < x->batch; ++b) {
    const int64_t r = (int64_t)b * n_heads;
    hipError_t e = launch_build_vs(view(x, b), hl, last_q, nv, ns, out->v_idx + r * nv,
                                   out->s_idx + r * ns, out->cover + r * ns * 2,
                                   out->cover_bits + r * out->cover_words, out->counts + r * 4,
                                   out->cover_words, ws, st);
    if (e != hipSuccess) return MINF_ERR_HIP;
  }
  return MINF_OK;
}

minf_status minf_build_vs_index(const minf_qkv *x, const int32_t *heads, int32_t n_heads,
                                int32_t last_q, int32_t nv, int32_t ns, int32_t block,
                                minf_vs_index *out, void *ws, size_t ws_bytes, void *hip_stream) {
  return build_vs_common(x, heads, n_heads, last_q, nv, ns, block, out, ws, ws_bytes, false, hip_stream);
}

minf_status minf_build_vs_index_noalloc(const minf_qkv *x, const int32_t *heads, int32_t n_heads,
                                        int32_t last_q, int32_t nv, int32_t ns, int32_t block,
                                        minf_vs_index *out, void *hip_stream) {
  return build_vs_common(x, heads, n_heads, last_q, nv, ns, block, out, nullptr, 0, true, hip_stream);
}

minf_status minf_vs_index_from_lines(int32_t seq_len, int32_t rows, minf_vs_index *idx, void *hip_stream) {
  if (!idx || !idx->v_idx || !idx->s_idx || !idx->cover || !idx->cover_bits || !idx->counts) return MINF_ERR_NULL;
  if (seq_len < MINF_BLOCK || seq_len % MINF_BLOCK != 0 || rows < 1) return MINF_ERR_SHAPE;
  if (idx->block != MINF_BLOCK) return MINF_ERR_UNSUPPORTED;
  if (idx->nv < 1 || idx->ns < 1) return MINF_ERR_BUDGET;
  if (idx->cover_words < minf_vs_cover_words(seq_len)) return MINF_ERR_SHAPE;
  return from_hip(launch_vs_lines(seq_len, rows, idx->nv, idx->ns, idx->s_idx, idx->cover, idx->cover_bits,
                                  idx->counts, idx->cover_words, static_cast<hipStream_t>(hip_stream)));
}

minf_status minf_build_bs_index(const minf_qkv *x, const int32_t *heads, int32_t n_heads,
                                int32_t block, int32_t topk, minf_bs_index *out, void *ws,
                                size_t ws_bytes, void *hip_stream) {
  minf_status s = check_qkv(x, false);
  if (s != MINF_OK) return s;
  HeadList hl;
  if ((s = check_heads(x, heads, n_heads, hl)) != MINF_OK) return s;
  if (block != MINF_BLOCK) return MINF_ERR_UNSUPPORTED;
  if (topk < 1) return MINF_ERR_BUDGET;
  if (!out || !out->blk_idx || !out->blk_cnt) return MINF_ERR_NULL;
  if (out->topk != topk || out->block != block) return MINF_ERR_BUDGET;
  const size_t need = bs_index_ws_bytes(x->seq_len, n_heads, topk);
  if (!ws || ws_bytes < need) return MINF_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) return MINF_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int64_t NB = x->seq_len / MINF_BLOCK;
  for (int b = 0; b < x->batch; ++b) {
    const int64_t r = (int64_t)b * n_heads;
    hipError_t e = launch_build_bs(view(x, b), hl, topk, out->blk_idx + r * NB * topk,
                                   out->blk_cnt + r * NB, out->order ? out->order + r * NB : nullptr, ws, st);
    if (e != hipSuccess) return MINF_ERR_HIP;
  }
  return MINF_OK;
}

minf_status minf_ashape_attn(const minf_qkv *x, const int32_t *heads, int32_t n_heads,
                             int32_t n_init, int32_t n_local, void *hip_stream) {
  minf_status s = check_qkv(x, true);
  if (s != MINF_OK) return s;
  HeadList hl;
  if ((s = check_heads(x, heads, n_heads, hl)) != MINF_OK) return s;
  if (n_init < 0 || n_local < 1) return MINF_ERR_BUDGET;
  n_init = n_init < x->seq_len ? n_init : x->seq_len;
  n_local = n_local < x->seq_len ? n_local : x->seq_len;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  for (int b = 0; b < x->batch; ++b) {
    hipError_t e = launch_ashape(view(x, b), hl, n_init, n_local, st);
    if (e != hipSuccess) return MINF_ERR_HIP;
  }
  return MINF_OK;
}

minf_status minf_dense_attn(const minf_qkv *x, const int32_t *heads, int32_t n_heads,
                            void *hip_stream) {
  if (!x) return MINF_ERR_NULL;
  return minf_ashape_attn(x, heads, n_heads, 0, x->seq_len > 0 ? x->seq_len : 1, hip_stream);
}

minf_status minf_vs_attn(const minf_qkv *x, const int32_t *heads, int32_t n_heads,
                         const minf_vs_index *idx, void *hip_stream) {
  minf_status s = check_qkv(x, true);
  if (s != MINF_OK) return s;
  HeadList hl;
  if ((s = check_heads(x, heads, n_heads, hl)) != MINF_OK) return s;
  if (!idx || !idx->v_idx || !idx->cover || !idx->cover_bits || !idx->counts) return MINF_ERR_NULL;
  if (idx->block != MINF_BLOCK) return MINF_ERR_UNSUPPORTED;
  if (idx->nv < 1 || idx->ns < 1) return MINF_ERR_BUDGET;
  if (idx->cover_words < minf_vs_cover_words(x->seq_len)) return MINF_ERR_SHAPE;
  // the gathered verticals are addressed with 32-bit byte offsets from the head's first row
  if ((uint64_t)x->seq_len * (uint64_t)x->k_stride[2] * 2u >= (1ull << 32) ||
      (uint64_t)x->seq_len * (uint64_t)x->v_stride[2] * 2u >= (1ull << 32))
    return MINF_ERR_SHAPE;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  for (int b = 0; b < x->batch; ++b) {
    const int64_t r = (int64_t)b * n_heads;
    hipError_t e = launch_vs(view(x, b), hl, idx->v_idx + r * idx->nv, idx->cover + r * idx->ns * 2,
                             idx->cover_bits + r * idx->cover_words, idx->counts + r * 4, idx->nv,
                             idx->ns, idx->cover_words, st);
    if (e != hipSuccess) return MINF_ERR_HIP;
  }
  return MINF_OK;
}

minf_status minf_bs_attn(const minf_qkv *x, const int32_t *heads, int32_t n_heads,
                         const minf_bs_index *idx, void *hip_stream) {
  minf_status s = check_qkv(x, true);
  if (s != MINF_OK) return s;
  HeadList hl;
  if ((s = check_heads(x, heads, n_heads, hl)) != MINF_OK) return s;
  if (!idx || !idx->blk_idx || !idx->blk_cnt) return MINF_ERR_NULL;
  if (idx->block != MINF_BLOCK) return MINF_ERR_UNSUPPORTED;
  if (idx->topk < 1) return MINF_ERR_BUDGET;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int64_t NB = x->seq_len / MINF_BLOCK;
  for (int b = 0; b < x->batch; ++b) {
    const int64_t r = (int64_t)b * n_heads;
    hipError_t e = launch_bs(view(x, b), hl, idx->blk_idx + r * NB * idx->topk, idx->blk_cnt + r * NB,
                             idx->order ? idx->order + r * NB : nullptr, idx->topk, st);
    if (e != hipSuccess) return MINF_ERR_HIP;
  }
  return MINF_OK;
}

minf_status minf_vs_bs_attn(const minf_qkv *x, const int32_t *vs_heads, int32_t n_vs, const minf_vs_index *vs,
                            const int32_t *bs_heads, int32_t n_bs, const minf_bs_index *bs, void *hip_stream) {
  minf_status s = check_qkv(x, true);
  if (s != MINF_OK) return s;
  HeadList hv, hb;
  if ((s = check_heads(x, vs_heads, n_vs, hv)) != MINF_OK) return s;
  if ((s = check_heads(x, bs_heads, n_bs, hb)) != MINF_OK) return s;
  if (!vs || !vs->v_idx || !vs->cover || !vs->cover_bits || !vs->counts) return MINF_ERR_NULL;
  if (!bs || !bs->blk_idx || !bs->blk_cnt) return MINF_ERR_NULL;
  if (vs->block != MINF_BLOCK || bs->block != MINF_BLOCK) return MINF_ERR_UNSUPPORTED;
  if (vs->nv < 1 || vs->ns < 1 || bs->topk < 1) return MINF_ERR_BUDGET;
  if (vs->cover_words < minf_vs_cover_words(x->seq_len)) return MINF_ERR_SHAPE;
  if ((uint64_t)x->seq_len * (uint64_t)x->k_stride[2] * 2u >= (1ull << 32) ||
      (uint64_t)x->seq_len * (uint64_t)x->v_stride[2] * 2u >= (1ull << 32))
    return MINF_ERR_SHAPE;
  // a head in both lists would be written by two work items
  for (int i = 0; i < n_vs; ++i)
    for (int j = 0; j < n_bs; ++j)
      if (vs_heads[i] == bs_heads[j]) return MINF_ERR_SHAPE;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int64_t NB = x->seq_len / MINF_BLOCK;
  for (int b = 0; b < x->batch; ++b) {
    const int64_t rv = (int64_t)b * n_vs, rb = (int64_t)b * n_bs;
    hipError_t e = launch_vs_bs(view(x, b), hv, vs->v_idx + rv * vs->nv, vs->cover + rv * vs->ns * 2,
                                vs->cover_bits + rv * vs->cover_words, vs->counts + rv * 4, vs->nv, vs->ns,
                                vs->cover_words, hb, bs->blk_idx + rb * NB * bs->topk, bs->blk_cnt + rb * NB,
                                bs->order ? bs->order + rb * NB : nullptr, bs->topk, st);
    if (e != hipSuccess) return MINF_ERR_HIP;
  }
  return MINF_OK;
}

}  // extern "C"
