// Device-side building blocks shared by the attention and index kernels:
// MFMA vector types, the LDS tile layout and the global -> LDS tile fetch.
#ifndef MINF_MFMA_TILE_H_
#define MINF_MFMA_TILE_H_

#include "minf_internal.h"

namespace minf {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int D = 128;         // head dim
constexpr int BQ = 64;         // query rows per wave (one paper block)
constexpr int BK = 64;         // keys per tile
constexpr int ROW_BYTES = 256; // one K or V row in LDS (128 bf16)
constexpr int KEY_NONE = 0x7fffffff;   // gathered column that must not be attended
constexpr int TILE_BYTES = BK * ROW_BYTES;       // one 64-row K or V tile in LDS
constexpr int HALF_BYTES = TILE_BYTES / 2;       // 32 rows

// Completion of direct global -> LDS loads is awaited by hand (they are issued from
// inline assembly, the compiler does not track them).
#define MINF_WAIT_VMCNT(n) asm volatile("s_waitcnt vmcnt(" #n ")" ::: "memory")

#define MINF_GPTR(p) ((__attribute__((address_space(1))) void *)(p))
#define MINF_LPTR(p) ((__attribute__((address_space(3))) void *)(p))

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Moves a wave-uniform value that the compiler computed on the vector ALU (an
// integer division, say) into a scalar register, so that what is derived from
// it (base pointers) is scalar work.  The builtin alone is folded away when the
// compiler can prove uniformity and the value then stays in vector registers.
// The compiler does not look inside the block, so the wait states that gfx950
// requires between a vector write of v and v_readfirstlane reading it, and
// between the scalar result and a memory instruction using it, are spelt out.
__device__ inline int to_sgpr(int v) {
  int s;
  asm("s_nop 3\n\tv_readfirstlane_b32 %0, %1\n\ts_nop 4" : "=s"(s) : "v"(v));
  return s;
}

// Row permutation applied when K rows are read as MFMA A-operand rows: MFMA
// row m = 16t + 8u + 4h + w holds key 16t + 8h + 4u + w.  With it, the 8
// accumulator registers 8t..8t+7 of lane-half h hold 8 consecutive keys
// (16t + 8h .. +7), which is what a B operand of the next MFMA must hold.
__device__ inline int perm_row(int m) { return (m & ~12) | ((m & 4) << 1) | ((m & 8) >> 1); }

// ---------------------------------------------------------------------------
// LDS tile layout.  A K or V tile is ROWS rows of 256 B, row-major, with the
// 16-byte chunk c of row r stored at chunk position c ^ f(r & 15), where f swaps
// the two 2-bit halves of its argument.  Any bijection f spreads the 16 rows
// that 16 lanes read at one column (K operand, ds_read_b128) over all 64
// banks; this one also sends 4 consecutive rows to 4 different 64-byte
// quarters of the bank window, which the transposing V read needs (each half
// wave touches 4 keys x 64 bytes).  The tile is filled by direct global -> LDS loads
// (global_load_lds_dwordx4: lane L's 16 bytes land at base + 16 L, so one
// instruction fills one 1 KiB block = 4 rows and every lane fetches the chunk
// that belongs at its position); no VGPRs and no LDS store instructions are
// spent on staging.
// ---------------------------------------------------------------------------
__device__ inline int swz_f(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }
__device__ inline int swz_byte(int r, int c16) { return r * ROW_BYTES + ((c16 ^ swz_f(r)) << 4); }

// One direct global -> LDS load of 16 bytes per lane: lane L's bytes land at
// LDS byte address lds_addr + 16 L (lds_addr wave-uniform).  Written as inline
// assembly so that the compiler does not serialise later LDS reads of OTHER
// tiles behind it; completion is awaited explicitly with s_waitcnt vmcnt.
__device__ inline void dma16(const void *g, unsigned lds_addr) {
  const unsigned a = __builtin_amdgcn_readfirstlane(lds_addr);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :: "v"(g), "s"(a) : "memory");
}

__device__ inline unsigned lds_addr_of(const void *p) {
  return (unsigned)(size_t)(__attribute__((address_space(3))) const char *)p;
}

// Same, with the address split into a wave-uniform 64-bit base (SGPR pair) and a
// per-lane 32-bit byte offset: no vector ALU work per load.
__device__ inline void dma16_su(const void *ubase, unsigned voff, unsigned lds_addr) {
  const unsigned long long b = (unsigned long long)ubase;
  const unsigned blo = __builtin_amdgcn_readfirstlane((unsigned)b);
  const unsigned bhi = __builtin_amdgcn_readfirstlane((unsigned)(b >> 32));
  const unsigned long long bs = ((unsigned long long)bhi << 32) | blo;
  const unsigned a = __builtin_amdgcn_readfirstlane(lds_addr);
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(voff), "s"(bs), "s"(a) : "memory");
}

// Per-lane constants of the tile fetch.  Row r = 4 blk + rl (rl = lane / 16) of a
// tile lives in 1 KiB block blk; lane L holds chunk position cpos = L % 16, i.e.
// the logical chunk cpos ^ f(r) = (cpos ^ (rl << 2)) ^ (blk & 3).  So the byte
// offset of lane L's source inside block blk is
//   4 blk row_bytes  (wave-uniform)  +  voff[blk & 3]  (per lane, fixed for the kernel).
struct DmaLane {
  unsigned voff[4];
};
__device__ inline void dma_lane_init(DmaLane &d, int64_t stride, int lane) {
  const unsigned rl = lane >> 4, cpos = lane & 15, row_bytes = (unsigned)stride * 2u;
#pragma unroll
  for (int j = 0; j < 4; ++j) d.voff[j] = rl * row_bytes + (((cpos ^ (rl << 2)) ^ j) << 4);
}

// Fetch ROWS rows into the tile at `tile` (LDS).  NW waves cooperate: wave w
// issues blocks w ROWS/4/NW, ... (consecutive).  CONTIG: rows are keys kbase + r; rows outside
// [0, N) are clamped (the caller masks them); a step that lies wholly inside
// [0, N) -- the common case -- takes the uniform-base form, which costs scalar
// ALU work only.  Otherwise keys come from cols[r] in LDS (KEY_NONE reads row 0
// and is masked by the caller).  stride * 2 * 64 must fit 32 bits.
template <int NW, int ROWS, bool CONTIG>
__device__ inline void dma_rows(const bf16_t *g, int64_t stride, const DmaLane &dl, int kbase,
                                const int *cols, int N, char *tile, int wave, int lane) {
  const unsigned base = lds_addr_of(tile);
  if (CONTIG && kbase >= 0 && kbase + ROWS <= N) {
    const bf16_t *ubase = g + (int64_t)kbase * stride;
#pragma unroll
    for (int i = 0; i < ROWS / 4 / NW; ++i) {
      const int blk = wave * (ROWS / 4 / NW) + i;    // ROWS / 4 / NW is a multiple of 4: blk & 3 == i & 3
      const unsigned voff = dl.voff[i & 3];
      dma16_su(ubase + (int64_t)(4 * blk) * stride, voff, base + blk * 1024);
    }
    return;
  }
  const int rl = lane >> 4, cpos = lane & 15;
#pragma unroll
  for (int i = 0; i < ROWS / 4 / NW; ++i) {
    const int blk = wave * (ROWS / 4 / NW) + i;
    const int r = 4 * blk + rl;
    const int c = cpos ^ swz_f(r);
    int key;
    if (CONTIG) {
      key = min(max(kbase + r, 0), N - 1);
    } else {
      key = cols[r];
      key = key == KEY_NONE ? 0 : key;
    }
    dma16(g + (int64_t)key * stride + c * 8, base + blk * 1024);
  }
}

// Per-lane byte offsets, inside a tile, of the MFMA A operands.
//  K (S^T = K Q^T): lane (n = lane%32, h = lane/32), k step ks reads the 16 B
//    chunk 2ks + h of row perm_row(n) (+ 32 rows per key block).
//  V (O^T += V^T P^T): the operand wants 8 consecutive keys of one d column per
//    lane while V rows hold d contiguous; ds_read_b64_tr_b16 transposes 4 keys
//    x 16 d inside each group of 16 lanes: lane 4j + c of a group addresses
//    V[key0 + j][d0 + 4c .. +3] and lane i receives V[key0 + 0..3][d0 + i].
struct LaneOfs {
  int k[8];        // [ks]
  int v[4][2];     // [d block][half: keys +0..3 / +4..7], add (32mb + 16t) * 256
};

__device__ inline void lane_offsets(LaneOfs &lo, int lane) {
  const int n = lane & 31, h = lane >> 5, prow = perm_row(n);
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) lo.k[ks] = swz_byte(prow, 2 * ks + h);
  const int msub = (lane >> 4) & 1, l16 = lane & 15, j = l16 >> 2, c = l16 & 3;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int key = 8 * h + 4 * half + j;
      const int c16 = 4 * db + 2 * msub + (c >> 1);
      lo.v[db][half] = swz_byte(key, c16) + (c & 1) * 8;
    }
}

__device__ inline bf16x8 lds_read_k(const char *tileK, int ofs) {
  return *reinterpret_cast<const bf16x8 *>(tileK + ofs);
}

__device__ inline bf16x8 lds_read_vt(const char *tileV, int ofs0, int ofs1) {
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)MINF_LPTR(tileV + ofs0));
  const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)MINF_LPTR(tileV + ofs1));
  const s16x8 w = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, w);
}

}  // namespace minf
#endif
