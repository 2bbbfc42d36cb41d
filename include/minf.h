/*
 * minf.h -- C ABI of the MI355X (gfx950) dynamic sparse prefill attention library.
 *
 * The library implements the online part of MInference 1.0 (arXiv 2407.02490):
 *   - sparse index construction for Vertical-Slash heads (Alg. 2, first three
 *     steps plus "sparseformat"; App. C.4.2) and Block-Sparse heads (Alg. 3),
 *   - causal sparse attention A(M) = softmax(QK^T/sqrt(d) - c(1-M)) V (Eq. 1)
 *     for the A-shape, Vertical-Slash and Block-Sparse masks M (Section 3.2,
 *     App. C.4), plus dense causal attention as the comparison kernel.
 *
 * General rules
 *   - Every pointer inside minf_qkv, minf_vs_index, minf_bs_index and every
 *     `ws` argument is a DEVICE pointer owned by the caller.  `heads` arrays
 *     and the structs themselves live on the HOST.
 *   - The library never allocates, frees or synchronises.  All work is
 *     enqueued on `hip_stream` (a hipStream_t passed as void*; NULL = the
 *     default stream).  Index structs written by minf_build_* may be consumed
 *     by the attention calls on the same stream without a host round trip.
 *   - Arguments are validated on the host before anything is enqueued: with
 *     any status other than MINF_OK and MINF_ERR_HIP nothing was launched.
 *     MINF_ERR_HIP means the runtime refused a launch; with batch > 1 the
 *     launches of earlier batch elements may already be enqueued then.
 *   - Layout: q [batch, n_q_heads, seq_len, head_dim], k/v [batch, n_kv_heads,
 *     seq_len, head_dim], o like q; bf16; head_dim contiguous; strides in
 *     elements for (batch, head, token).  Query head h reads KV head
 *     h / (n_q_heads / n_kv_heads) (grouped-query attention).
 *   - This version requires head_dim == 128, block == 64, seq_len % 64 == 0,
 *     n_heads <= MINF_MAX_HEADS per call.
 *   - The head -> pattern assignment (the output of the paper's offline
 *     search, Section 3.2) is expressed by which call a head id is passed to;
 *     budgets are per call.  Each attention call writes O only for its heads.
 */
#ifndef MINF_H_
#define MINF_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MINF_MAX_HEADS 128
#define MINF_BLOCK 64

typedef enum {
  MINF_OK = 0,
  MINF_ERR_NULL = 1,        /* a required pointer is NULL                         */
  MINF_ERR_SHAPE = 2,       /* unsupported head_dim / seq_len / strides / heads   */
  MINF_ERR_BUDGET = 3,      /* nv, ns, topk, last_q, n_init, n_local out of range */
  MINF_ERR_WORKSPACE = 4,   /* ws is NULL or smaller than minf_*_workspace_bytes  */
  MINF_ERR_UNSUPPORTED = 5, /* block != 64 and the like                           */
  MINF_ERR_HIP = 6          /* the HIP runtime refused a launch                   */
} minf_status;

typedef struct {
  const void *q, *k, *v;    /* device, bf16                                        */
  void *o;                  /* device, bf16, same shape as q                       */
  int64_t q_stride[3], k_stride[3], v_stride[3], o_stride[3]; /* batch, head, token */
  int32_t batch, n_q_heads, n_kv_heads, seq_len, head_dim;
  float softmax_scale;      /* 0 -> 1/sqrt(head_dim)                               */
} minf_qkv;

/*
 * Vertical-Slash index of n_heads heads (Alg. 2: i_v, i_s; Alg. 4's role).
 * Row r of every array belongs to heads[r] of the build call (batch-major:
 * row = batch_index * n_heads + r).
 *   v_idx  [rows, nv]   key positions of the kept vertical lines, ascending
 *   s_idx  [rows, ns]   diagonal offsets i-j of the kept slash lines, ascending
 *   cover  [rows, ns, 2] the slash lines as merged offset runs [t0, t1), ascending
 *                       and disjoint: for the 64-row query block starting at row
 *                       q0 a run permits the keys j = q0 - t, t0 <= t < t1 (j >= 0,
 *                       j <= i).  This is the union over the kept slashes o of
 *                       the 64 x 64 tile whose main diagonal is slash o
 *                       (App. C.4.2); it does not depend on the query block, so
 *                       it is stored once per head instead of per block row.
 *   cover_bits [rows, cover_words] bit (t + 64) set iff offset t is in a run;
 *                       used to drop verticals already inside a slash tile.
 *   counts [rows, 4]    {n_v, n_s, n_cover, 0}: entries actually valid
 *                       (nv, ns clamp to seq_len).
 * cover_words must be >= minf_vs_cover_words(seq_len).
 */
typedef struct {
  int32_t *v_idx;
  int32_t *s_idx;
  int32_t *cover;
  uint32_t *cover_bits;
  int32_t *counts;
  int32_t nv, ns, block, cover_words;
} minf_vs_index;

/*
 * Block-Sparse index (Alg. 3: i_b).
 *   blk_idx [rows, NB, topk] kept key-block ids of query block b, ascending;
 *                            entries past blk_cnt are -1
 *   blk_cnt [rows, NB]       min(topk, b + 1)
 *   order   [rows, NB]       the order in which minf_bs_attn takes the query
 *                            blocks of a head: a permutation of 0 .. NB-1, or
 *                            NULL for 0, 1, 2, ...  It has no influence on the
 *                            result.  minf_build_bs_index sorts the query
 *                            blocks by their first kept key block (then by
 *                            block id): query blocks that attend the same key
 *                            blocks (Section 2.2: the blocks cluster) then run
 *                            at the same time on the same part of the chip and
 *                            find each other's K/V tiles in its cache (up to
 *                            32768 blocks = 2M tokens; longer sequences get the
 *                            natural order).  A caller that fills the index
 *                            itself may leave it NULL.
 */
typedef struct {
  int32_t *blk_idx;
  int32_t *blk_cnt;
  int32_t *order;
  int32_t topk, block;
} minf_bs_index;

const char *minf_status_string(minf_status s);

/* Number of 32-bit words per head of minf_vs_index.cover_bits. */
int32_t minf_vs_cover_words(int32_t seq_len);

/* Workspace sizes in bytes (0 on invalid arguments).  The Block-Sparse build needs the pooled K
 * only (512 bytes per head and 64-token block) when topk <= 112 and the sequence has fewer than
 * 65536 blocks: pooling of Q, block logits and selection are then fused and neither the pooled Q
 * nor a logit is stored.  Larger budgets also keep the pooled Q and stage the logits of a few
 * heads at a time: up to 2 GiB more. */
size_t minf_vs_index_workspace_bytes(const minf_qkv *x, int32_t n_heads, int32_t last_q);
size_t minf_bs_index_workspace_bytes(const minf_qkv *x, int32_t n_heads, int32_t topk);

/*
 * Alg. 2, index part.  For each listed head: A_hat = softmax(Q[-last_q:] K^T
 * / sqrt(d) + causal), column sums and diagonal sums of A_hat, exact top-nv /
 * top-ns (ties to the lower index), ascending sort, merge of the slash tiles
 * into offset runs.  Logits are bf16 MFMA products with fp32 accumulation;
 * softmax and the sums are fp32 in a fixed order (bit-reproducible).
 * 1 <= last_q <= 64; nv, ns >= 1 (the kernels need at least one vertical and
 * one slash, cf. App. D.3); block must be 64.
 */
minf_status minf_build_vs_index(const minf_qkv *x, const int32_t *heads, int32_t n_heads,
                                int32_t last_q, int32_t nv, int32_t ns, int32_t block,
                                minf_vs_index *out, void *ws, size_t ws_bytes,
                                void *hip_stream);

/*
 * minf_build_vs_index for callers that cannot allocate device memory and have
 * no workspace to pass: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, checks and results as
 * minf_build_vs_index, but the line scores and softmax statistics go to a
 * scratch array that is part of the library (a file-scope device array of
 * MINF_NOALLOC_SCRATCH_BYTES bytes per GPU, held until the process ends)
 * instead of `ws`.  Allocates nothing, frees nothing, synchronises nothing.
 * Inputs whose workspace need (minf_vs_index_workspace_bytes) exceeds
 * MINF_NOALLOC_SCRATCH_BYTES are refused with MINF_ERR_WORKSPACE; with
 * batch > 1 the batch elements use the array one after the other on the
 * stream.  All calls on one GPU share that GPU's array: calls that overlap
 * in time on one GPU (different streams, different threads) race; nothing in
 * the array needs clearing between calls (every word that is read was
 * written by the same call).  The array's device address is looked up on the
 * first call on each device (MINF_ERR_HIP if the runtime refuses).
 */
#define MINF_NOALLOC_SCRATCH_BYTES (96u << 20)   /* 32 heads at 128K tokens need 74 MiB */
minf_status minf_build_vs_index_noalloc(const minf_qkv *x, const int32_t *heads, int32_t n_heads,
                                        int32_t last_q, int32_t nv, int32_t ns, int32_t block,
                                        minf_vs_index *out, void *hip_stream);

/*
 * The "sparseformat" step alone (Alg. 2; Alg. 4's role, App. C.4.2) for lines
 * the caller chose: the static-index use of the attention call (Section 4,
 * ablation "Ours w/ static").  On entry, for every row r < rows of idx:
 * v_idx[r, 0 .. n_v) holds the kept vertical positions and s_idx[r, 0 .. n_s)
 * the kept slash offsets, both ascending, distinct and inside [0, seq_len),
 * with counts[r] = {n_v, n_s, *, *} (device memory, n_v <= idx->nv,
 * n_s <= idx->ns).  Fills cover, cover_bits and counts[r][2..3] on the stream;
 * v_idx and s_idx are left as they are.  Offsets outside [0, seq_len) are
 * clamped into it.
 */
minf_status minf_vs_index_from_lines(int32_t seq_len, int32_t rows, minf_vs_index *idx,
                                     void *hip_stream);

/*
 * Alg. 3, index part.  Mean-pools Q and K over 64-token blocks (fp32), forms
 * the block logits Q_hat K_hat^T / sqrt(d) for c <= b in fp32 and keeps, per
 * query block, the min(topk, b+1) largest (softmax is monotone per row, so
 * it is not applied).  topk >= 1; block must be 64.  If out->order is not
 * NULL it receives the processing order of the query blocks (see
 * minf_bs_index).
 */
minf_status minf_build_bs_index(const minf_qkv *x, const int32_t *heads, int32_t n_heads,
                                int32_t block, int32_t topk, minf_bs_index *out,
                                void *ws, size_t ws_bytes, void *hip_stream);

/*
 * A-shape attention (Section 2.2; "1k global + 4k local", Section 4): query i
 * attends key j iff j <= i and (j < n_init or i - j < n_local), element exact.
 * n_init >= 0, n_local >= 1.
 */
minf_status minf_ashape_attn(const minf_qkv *x, const int32_t *heads, int32_t n_heads,
                             int32_t n_init, int32_t n_local, void *hip_stream);

/*
 * Vertical-Slash attention (Alg. 2 last steps, Alg. 5): per 64-row query block
 * the keys of the slash runs, then the kept verticals that are causal and not
 * already inside a run, gathered into dense steps.  Every permitted key is
 * attended exactly once; a row with no permitted key gives zeros.
 * Row r of idx belongs to heads[r].  The gathered verticals are addressed with
 * 32-bit byte offsets: seq_len * k_stride[2] * 2 and seq_len * v_stride[2] * 2
 * must be below 2^32 (MINF_ERR_SHAPE otherwise; e.g. a fused token-major QKV
 * buffer of 1M tokens with 16 or more heads per token is refused).
 */
minf_status minf_vs_attn(const minf_qkv *x, const int32_t *heads, int32_t n_heads,
                         const minf_vs_index *idx, void *hip_stream);

/*
 * Block-Sparse attention (Alg. 3 last steps, App. C.4.1): per 64-row query
 * block the listed 64-key blocks, element causal.  Block ids outside
 * [0, NB) are ignored.
 */
minf_status minf_bs_attn(const minf_qkv *x, const int32_t *heads, int32_t n_heads,
                         const minf_bs_index *idx, void *hip_stream);

/*
 * Vertical-Slash and Block-Sparse heads of one layer in a single launch (the
 * layers of the paper's models mix the patterns: Section 3.2, App. E).  Same
 * arguments, checks and results (bit for bit) as minf_vs_attn on vs_heads
 * followed by minf_bs_attn on bs_heads; a head must not be in both lists
 * (MINF_ERR_SHAPE).  The work items of the two patterns are interleaved four
 * to one so that every part of the chip holds both kinds at once.  Measured
 * slower than the two separate calls on the mixed 1M-token layer (the
 * patterns disturb each other's cache reuse); provided as the measured
 * alternative.
 */
minf_status minf_vs_bs_attn(const minf_qkv *x, const int32_t *vs_heads, int32_t n_vs, const minf_vs_index *vs,
                            const int32_t *bs_heads, int32_t n_bs, const minf_bs_index *bs, void *hip_stream);

/* Dense causal attention with the same kernels: the speedup baseline. */
minf_status minf_dense_attn(const minf_qkv *x, const int32_t *heads, int32_t n_heads,
                            void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MINF_H_ */
