// Exact re-decision of the tokens at the selection threshold, shared by the standalone refinement kernel and by the
// fused select+refine kernel so that both take bit-identical decisions.
#pragma once
#include "common.hpp"

namespace obf {

// eight consecutive elements as floats, one 16-byte (bf16) or two 16-byte (fp32) loads; p must be 16-byte aligned
__device__ __forceinline__ void load8(const uint16_t* p, float (&o)[8]) {
  const uint4 v = *(const uint4*)p;
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) { o[2 * i] = __uint_as_float(w[i] << 16); o[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u); }
}
__device__ __forceinline__ void load8(const float* p, float (&o)[8]) {
  const float4 a = *(const float4*)p, b = *(const float4*)(p + 4);
  o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
}

// Exact (double) attention mass of each band token: one wave per token, lanes over the query rows, fixed
// summation order (row stride 64 per lane, then a butterfly over the lanes).
template <typename T, int WAVES>
__device__ __forceinline__ void rescore_band(const T* __restrict__ Kh, const T* __restrict__ Qh,
                                             const double* __restrict__ lse, int d, int R, const int* band, int nband,
                                             double* band_score) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const double scale = 1.0 / sqrt((double)d);
  for (int b = wave; b < nband; b += WAVES) {
    const T* kr = Kh + (size_t)band[b] * d;
    double part = 0.0;
    for (int r = lane; r < R; r += 64) {
      const T* qr = Qh + (size_t)r * d;
      double acc = 0.0;
#pragma unroll 4
      for (int c = 0; c < d; c += 8) {                  // head_dim is a multiple of 8; same element order as a scalar loop
        float qv[8], kv[8];
        load8(qr + c, qv);
        load8(kr + c, kv);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc = fma((double)qv[e], (double)kv[e], acc);
      }
      part += exp(acc * scale - lse[r]);
    }
    for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off);
    if (lane == 0) band_score[b] = part;
  }
}

// Thread u < nband: is band token u among the nkb best (exact score descending, index ascending; band[] is ascending)?
__device__ __forceinline__ int band_keeps(const double* band_score, int nband, int nkb, int u) {
  const double mine = band_score[u];
  int rank = 0;
  for (int v = 0; v < nband; ++v) {
    const double o = band_score[v];
    rank += (o > mine) || (o == mine && v < u);
  }
  return rank < nkb;
}

}  // namespace obf
