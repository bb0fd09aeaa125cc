// Staging of bf16 rows of width 128 for Gram products V^T V on the matrix cores (v_mfma_f32_32x32x16_bf16), shared by
// the kernels that form such products (the statistics of the deleted rows, the full-rank certificate of the retained
// rows).  An operand fragment of that instruction holds, per lane, eight consecutive k-entries of one row of the
// operand; for V^T V the k-index is the token, so a lane needs eight tokens of ONE column - the transpose of how
// rows lie in memory.  Rows therefore pass through LDS in this layout:
//   word [p][j] of a staged tile of 64 rows holds column j of rows 2p and 2p+1 (low / high half), row stride
//   GS_LDW words, so that a fragment (8 rows of one column) is four 32-bit reads from consecutive row pairs.
// A workgroup of NW waves moves a tile as 16-byte pieces (eight columns of one row): lane l of wave w handles, for
// q = 0 .. 16 / NW - 1, piece l % 16 of row 4 (w + NW q) + tl, tl = 2 ((l / 16) % 2) + l / 32.  Lanes l and l + 32 hold the
// two rows of a pair; one lane swap per word pair brings the partner row's words for four of the eight columns to
// each lane (the lower lane ends up with the piece's columns 0 - 3 of both rows, the upper lane with columns 4 - 7),
// two byte permutes interleave them, and one 16-byte LDS store places them.
#pragma once
#include "common.hpp"

namespace obf {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 gs_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float gs_f32x16;

constexpr int GS_D = 128;
constexpr int GS_TILE = 64;              // rows per staged tile
constexpr int GS_LDW = 136;              // staging stride in 32-bit words per row PAIR (the two lane halves, 4 pairs apart, use different banks)
constexpr int GS_STAGE_WORDS = (GS_TILE / 2) * GS_LDW;

union GsFrag { uint32_t w[4]; uint4 q; gs_bf16x8 v; };

// row within the tile that lane `lane` of wave `wave` moves in round q (NW waves per workgroup)
template <int NW>
__device__ __forceinline__ int gs_row(int wave, int lane, int q) { return 4 * (wave + NW * q) + ((lane >> 4) & 1) * 2 + (lane >> 5); }

// Stores the piece `src` (columns 8 pc .. 8 pc + 7 of tile row rl, held by this lane; the partner lane holds the other
// row of the pair) into the staged tile.  keep == 0 stages zeros instead (a row that must not enter the product).
__device__ __forceinline__ void gs_put(uint32_t* __restrict__ tile, int rl, int lane, uint4 src, bool keep) {
  const uint32_t mk = keep ? 0xffffffffu : 0u;
  const auto s0 = __builtin_amdgcn_permlane32_swap(src.x & mk, src.z & mk, false, false);   // [0]: even row, [1]: odd row
  const auto s1 = __builtin_amdgcn_permlane32_swap(src.y & mk, src.w & mk, false, false);
  uint4 wv;
  wv.x = __builtin_amdgcn_perm(s0[1], s0[0], 0x05040100u);
  wv.y = __builtin_amdgcn_perm(s0[1], s0[0], 0x07060302u);
  wv.z = __builtin_amdgcn_perm(s1[1], s1[0], 0x05040100u);
  wv.w = __builtin_amdgcn_perm(s1[1], s1[0], 0x07060302u);
  *(uint4*)(&tile[(rl >> 1) * GS_LDW + (lane & 15) * 8 + (lane >> 5) * 4]) = wv;
}

// The fragment of column block `col_words / 32` for k-step ks of a staged tile: rows 16 ks + 8 (lane / 32) .. + 7 of
// column col_words + lane % 32.  The order of the rows inside a fragment is the same for every column, which is all a
// product of two such fragments needs.
__device__ __forceinline__ void gs_frag(GsFrag& f, const uint32_t* __restrict__ tile, int ks, int lane, int col_words) {
  const uint32_t* p = tile + (ks * 8 + (lane >> 5) * 4) * GS_LDW + col_words + (lane & 31);
#pragma unroll
  for (int i = 0; i < 4; ++i) f.w[i] = p[i * GS_LDW];
}

}  // namespace obf
