// Device-side building blocks shared by the attention and index kernels:
// MFMA vector types, LDS tile geometry, global -> register -> LDS tile staging.
#ifndef MINF_MFMA_TILE_H_
#define MINF_MFMA_TILE_H_

#include "minf_internal.h"

namespace minf {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int D = 128;         // head dim
constexpr int BQ = 64;         // query rows per wave (one paper block)
constexpr int BK = 64;         // keys per tile
constexpr int K_PITCH = 136;   // bf16 per LDS row of a K tile (256 B + 16 B pad)
constexpr int VT_PITCH = 72;   // bf16 per LDS row of a V^T tile (128 B + 16 B pad)
constexpr int K_TILE = BK * K_PITCH;      // 8704 elements
constexpr int VT_TILE = D * VT_PITCH;     // 9216 elements
constexpr int STAGE = K_TILE + VT_TILE;   // 17920 elements = 35840 B
constexpr int KEY_NONE = 0x7fffffff;      // gathered column that must not be attended
constexpr int VCAP = 1024;                // compacted vertical columns held in LDS per round

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Row permutation applied when K rows are read as MFMA A-operand rows: MFMA
// row m = 16t + 8u + 4h + w holds key 16t + 8h + 4u + w.  With it, the 8
// accumulator registers 8t..8t+7 of lane-half h hold 8 consecutive keys
// (16t + 8h .. +7), which is what a B operand of the next MFMA must hold.
__device__ inline int perm_row(int m) { return (m & ~12) | ((m & 4) << 1) | ((m & 8) >> 1); }

struct WaveState {
  bf16x8 q[2][8];     // Q fragments: [query half nb][k step]: Q[32nb + n][16ks + 8h ..]
  f32x16 o[4][2];     // O^T accumulators: [d block][query half]
  float m[2];         // running max of the scaled logits (log2 domain) of query 32nb + n
  float l[2];         // this lane's share of the running row sum
};

// Element mask of a tile, as seen by one wave (all fields wave-uniform).
// A key is attended by query row i iff lo <= key < hi, key <= i and
// (key < n_init or key + n_local > i).
struct MaskP {
  int q0;             // first query row of the wave's block
  int lo, hi;
  int n_init, n_local;
};

template <int NT>
struct TileRegs {
  uint4 k[1024 / NT];
  uint4 v[1024 / NT];
};

// ---- tile fetch: global -> registers ------------------------------------
// CONTIG: keys kbase .. kbase+63 (clamped to [0, N-1]; out-of-range keys are
// masked by the caller).  Otherwise keys come from cols[0..63] in LDS
// (KEY_NONE entries read row 0).
template <int NT, bool CONTIG>
__device__ inline void tile_issue(TileRegs<NT> &r, const bf16_t *kh, const bf16_t *vh, int64_t k_st,
                                  int64_t v_st, int kbase, const int *cols, int N, int tid) {
#pragma unroll
  for (int i = 0; i < 1024 / NT; ++i) {
    int c = tid + NT * i;
    int row = c >> 4, col = c & 15;
    int key;
    if (CONTIG) {
      key = min(max(kbase + row, 0), N - 1);
    } else {
      key = cols[row];
      key = key == KEY_NONE ? 0 : key;
    }
    r.k[i] = *reinterpret_cast<const uint4 *>(kh + (int64_t)key * k_st + col * 8);
  }
#pragma unroll
  for (int i = 0; i < 256 / NT; ++i) {
    int u = tid + NT * i;
    int kq = u >> 4, col = u & 15;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int row = 4 * kq + j;
      int key;
      if (CONTIG) {
        key = min(max(kbase + row, 0), N - 1);
      } else {
        key = cols[row];
        key = key == KEY_NONE ? 0 : key;
      }
      r.v[4 * i + j] = *reinterpret_cast<const uint4 *>(vh + (int64_t)key * v_st + col * 8);
    }
  }
}

// ---- tile store: registers -> LDS (K row-major, V transposed) -------------
template <int NT>
__device__ inline void tile_store(const TileRegs<NT> &r, bf16_t *ldsK, bf16_t *ldsVt, int tid) {
#pragma unroll
  for (int i = 0; i < 1024 / NT; ++i) {
    int c = tid + NT * i;
    int row = c >> 4, col = c & 15;
    *reinterpret_cast<uint4 *>(ldsK + row * K_PITCH + col * 8) = r.k[i];
  }
#pragma unroll
  for (int i = 0; i < 256 / NT; ++i) {
    int u = tid + NT * i;
    int kq = u >> 4, col = u & 15;
    const uint4 &a = r.v[4 * i + 0], &b = r.v[4 * i + 1], &c = r.v[4 * i + 2], &d = r.v[4 * i + 3];
    const unsigned aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
    const unsigned cw[4] = {c.x, c.y, c.z, c.w}, dw[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      // dword w of a row holds d = 2w (low half) and 2w+1 (high half)
      uint2 lo, hi;
      lo.x = __builtin_amdgcn_perm(bw[w], aw[w], 0x05040100u);  // (a.lo, b.lo)
      lo.y = __builtin_amdgcn_perm(dw[w], cw[w], 0x05040100u);  // (c.lo, d.lo)
      hi.x = __builtin_amdgcn_perm(bw[w], aw[w], 0x07060302u);  // (a.hi, b.hi)
      hi.y = __builtin_amdgcn_perm(dw[w], cw[w], 0x07060302u);
      int dd = col * 8 + 2 * w;
      *reinterpret_cast<uint2 *>(ldsVt + dd * VT_PITCH + 4 * kq) = lo;
      *reinterpret_cast<uint2 *>(ldsVt + (dd + 1) * VT_PITCH + 4 * kq) = hi;
    }
  }
}

}  // namespace minf
#endif
