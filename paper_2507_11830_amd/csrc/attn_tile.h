// Tile-level building blocks shared by the prefill and decode attention kernels (gfx950).
//
// Orientation.  Scores are computed TRANSPOSED, S^T[kv][q] = K Q^T, with
// v_mfma_f32_32x32x16_bf16: K rows are the M side (A operand), query columns the N side
// (B operand).  A lane then owns ONE query column (lane & 31) and 16 key rows per 32-key
// block, so the softmax reductions over keys are in-register plus one exchange between the
// two wave halves.  The output is accumulated transposed as well, O^T[d][q] = V^T P^T:
// the fp32 score accumulator of a lane, packed to bf16, is directly the B operand of that
// second MFMA — P never goes through LDS.  The contraction index of the second MFMA (the key
// index) may be permuted freely as long as both operands agree; the V^T operand is fetched
// from the row-major V tile in LDS with ds_read_b64_tr_b16 in the row order the score
// accumulator dictates.
//
// MFMA 32x32x16 register layouts (checked on hardware):
//   A (32 x 16): lane l holds row l & 31, k = 8 * (l >> 5) + 0..7
//   B (16 x 32): lane l holds col l & 31, k = 8 * (l >> 5) + 0..7
//   C (32 x 32): lane l holds col l & 31, register r holds row 8 * (r / 4) + 4 * (l >> 5) + r % 4
#pragma once
#include "sp_common.h"

namespace sp {

template <int D>
struct TileGeom {
  static constexpr int kDSteps = D / 16;        // MFMA k-steps of the QK^T contraction
  static constexpr int kDBlocks = D / 32;       // 32-row blocks of O^T
};

// LDS is addressed through explicit address-space-3 pointers so every access is a ds_* op.
typedef __attribute__((address_space(3))) char lds_char;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((address_space(3))) bf16x8 lds_bf16x8;
typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
typedef __attribute__((address_space(3))) float lds_float;

// V^T operand for one (32-channel block, 16-key step): two transposing 8-byte reads.  `p` is
// this lane's address for the first of its 4 consecutive key rows (lane n of a 16-lane group
// supplies row n / 4 and 8-byte piece n % 4 of a 32-byte run of channels); the second group of
// 4 rows sits 8 rows (8 * rowbytes) further.  Row offsets that are multiples of 8 rows leave the
// swizzle of SwzTile unchanged, so callers add them to a precomputed lane address.
__device__ __forceinline__ bf16x8 lds_read_vt(const lds_char *p, int rowbytes) {
  union {
    struct { s16x4 a, b; } s;
    bf16x8 v;
  } u;
  u.s.a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)p);
  u.s.b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + 8 * rowbytes));
  return u.v;
}

// Swizzled, unpadded tile layout.  Tiles are brought in with direct
// global -> LDS loads, which place the 64 lanes' 16-byte chunks back to back; padding between
// rows is therefore impossible, but every lane may fetch ANY global chunk, so the bank spread
// comes from a permutation instead: a tile is a sequence of 256-byte lines (one row at
// head_dim 128, two rows at 64) and chunk c of line L is stored in chunk slot c ^ g(L).
//   K tiles, g = L mod 16 (mod 8 at head_dim 64): the 16 consecutive rows that 16 lanes of a K
//   operand read (same chunk index) land in 16 different slots.
//   V tiles, g = 4 * (L mod 4) (4 * (L mod 2)): the 4 rows x 4 chunks that one half-wave of a
//   transposing V^T read touches land in 16 different slots.
template <int D>
struct SwzTile {
  static_assert(D == 128 || D == 64, "head_dim");
  static constexpr int kRowBytes = D * 2;
  __device__ static __forceinline__ int gk(int line) { return D == 128 ? (line & 15) : (line & 7); }
  __device__ static __forceinline__ int gv(int line) { return D == 128 ? ((line & 3) << 2) : ((line & 1) << 2); }
  // byte offset of 16-byte chunk `chunk` of tile row `row`
  template <bool V>
  __device__ static __forceinline__ int offset(int row, int chunk) {
    const int line = D == 128 ? row : row >> 1;
    const int c = D == 128 ? chunk : (((row & 1) << 3) | chunk);
    return line * 256 + ((c ^ (V ? gv(line) : gk(line))) << 4);
  }
};

// Exchange between the two 32-lane halves: returns the value held by lane ^ 32.
__device__ __forceinline__ float other_half(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  // lower half: r[1] is the upper lane's value; upper half: r[0] is the lower lane's value
  return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}

__device__ __forceinline__ bf16x8 pack8(const f32x16 &p, int r0) {
  union {
    bf16x2 h[4];
    bf16x8 v;
  } u;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    u.h[i] = __builtin_convertvector((f32x2){p[r0 + 2 * i], p[r0 + 2 * i + 1]}, bf16x2);
  return u.v;
}

// bf16 of what pack8 rounded away: p - float(hi).  Rows with only a few keys take their
// weights as hi + lo (two MFMA passes) so that the bf16 rounding of P does not eat into the
// output tolerance there; long rows average that rounding out and use hi alone.
__device__ __forceinline__ bf16x8 pack8_residual(const f32x16 &p, int r0, bf16x8 hi) {
  union {
    bf16x8 v;
    unsigned short s[8];
  } h;
  h.v = hi;
  union {
    bf16x2 q[4];
    bf16x8 v;
  } u;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float e0 = p[r0 + 2 * i] - __uint_as_float((uint32_t)h.s[2 * i] << 16);
    float e1 = p[r0 + 2 * i + 1] - __uint_as_float((uint32_t)h.s[2 * i + 1] << 16);
    u.q[i] = __builtin_convertvector((f32x2){e0, e1}, bf16x2);
  }
  return u.v;
}

// One 64-bit store of 4 consecutive bf16 outputs.
__device__ __forceinline__ void store4_bf16(void *dst, float a, float b, float c, float d) {
  union {
    bf16x2 h[2];
    u32x2 v;
  } u;
  u.h[0] = __builtin_convertvector((f32x2){a, b}, bf16x2);
  u.h[1] = __builtin_convertvector((f32x2){c, d}, bf16x2);
  *reinterpret_cast<u32x2 *>(dst) = u.v;
}

}  // namespace sp
