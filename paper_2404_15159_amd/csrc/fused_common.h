// Helpers shared by the bf16 MFMA versions of the per-pair stages (csrc/fused.hip: expert-grouped
// row tiles; csrc/fused_pg.hip: token tiles of one expert pair): lane roles, LDS tile access, fast sigmoid.
#pragma once
#include "common.h"

namespace mixlora {

typedef bf16_t bf16x4_t __attribute__((ext_vector_type(4)));

constexpr int FT_ROWS = 32;    // grouped rows per tile
constexpr int FT_WAVES = 4;

__device__ __forceinline__ bool fused_tile_rows(const int32_t *offs, int N, int b, int &e,
                                                int &row0, int &rows) {
  for (e = 0; e < N; e++) {
    const int lo = offs[e], hi = offs[e + 1];
    const int nt = (hi - lo + FT_ROWS - 1) / FT_ROWS;
    if (b < nt) {
      row0 = lo + b * FT_ROWS;
      rows = hi - row0 < FT_ROWS ? hi - row0 : FT_ROWS;
      return true;
    }
    b -= nt;
  }
  return false;
}

// v_exp_f32 + v_rcp_f32 (about 1 ulp each): far inside the bf16 tolerance, a tenth of the
// instructions of an IEEE division
__device__ __forceinline__ float fsigmoid(float v) { return __builtin_amdgcn_rcpf(1.f + __expf(-v)); }

// 8 consecutive fp32 -> bf16x8 (or zeros)
__device__ __forceinline__ bf16x8_t cvt8(const float *p, bool valid, float scale) {
  bf16x8_t o;
  if (valid) {
    const float4 a = *reinterpret_cast<const float4 *>(p);
    const float4 b = *reinterpret_cast<const float4 *>(p + 4);
    o[0] = (bf16_t)(a.x * scale); o[1] = (bf16_t)(a.y * scale);
    o[2] = (bf16_t)(a.z * scale); o[3] = (bf16_t)(a.w * scale);
    o[4] = (bf16_t)(b.x * scale); o[5] = (bf16_t)(b.y * scale);
    o[6] = (bf16_t)(b.z * scale); o[7] = (bf16_t)(b.w * scale);
  } else {
#pragma unroll
    for (int i = 0; i < 8; i++) o[i] = (bf16_t)0.f;
  }
  return o;
}

__device__ __forceinline__ bf16x8_t zero8() {
  bf16x8_t o;
#pragma unroll
  for (int i = 0; i < 8; i++) o[i] = (bf16_t)0.f;
  return o;
}

// ---- coalesced global traffic -------------------------------------------------------------------
// The MFMA result layout gives a lane 4-column runs of 32 different rows; used directly it would
// make every gathered load and every store an 8-byte piece.  The rank-r MFMA results therefore
// go through a small per-wave LDS tile ([32 rows][64 columns] bf16, padded pitch) instead, and all global
// traffic uses the "row-major" lane role: lane = (row 8p + lane/8, 8-column chunk lane%8), i.e.
// 16 bytes per lane and 128 contiguous bytes per row per instruction.  The activation (or
// gradient) tile is written back into the same LDS tile and read once more as MFMA first
// operand (index = row, contraction = columns) for the rank-r products with A_down / B^T.
// LDS operations of one wave execute in order, so the tiles need no workgroup barrier.
constexpr int FT_SB = 64;                 // columns per super-block
constexpr int FT_PITCH = FT_SB + 8;       // bf16 elements per LDS tile row (144 bytes)
constexpr int FT_TILE = FT_ROWS * FT_PITCH;

__device__ __forceinline__ bf16x8_t ld8(const bf16_t *p) { return *reinterpret_cast<const bf16x8_t *>(p); }

// write one 32x32 MFMA result block into an LDS tile at column offset cb32 (the LoRA scale is
// already in the per-row operand fragments)
__device__ __forceinline__ void tile_put(bf16_t *tile, int l31, int hi, int cb32, const f32x16_t &d) {
#pragma unroll
  for (int g = 0; g < 4; g++) {
    bf16x4_t v;
#pragma unroll
    for (int m = 0; m < 4; m++) v[m] = (bf16_t)d[g * 4 + m];
    *reinterpret_cast<bf16x4_t *>(tile + l31 * FT_PITCH + cb32 + 8 * g + 4 * hi) = v;
  }
}

}  // namespace mixlora
