// Cross-lane reductions on one 64-wide wave through DPP and lane-swap moves (no LDS traffic), and an LDS-only barrier.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace obf {

// The four in-row steps: lane ^ 1, lane ^ 2, mirror within 8, mirror within 16.  After them every lane of a
// 16-lane row holds the reduction over that row.
// Workgroup barrier that orders LDS traffic only: global stores still in flight (which nobody in the workgroup
// reads back) are not waited for, unlike with __syncthreads().
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

#define OBF_DPP_MOV(x, ctrl) ((uint32_t)__builtin_amdgcn_update_dpp(0, (int)(x), (ctrl), 0xF, 0xF, false))

// The value held by the next lower / next higher lane of the 64-lane wave (one DPP move each); lane 0 resp. lane 63
// gets an unspecified value.
__device__ __forceinline__ float wave_from_below(float v) { return __uint_as_float(OBF_DPP_MOV(__float_as_uint(v), 0x138)); }   // wave_shr:1
__device__ __forceinline__ float wave_from_above(float v) { return __uint_as_float(OBF_DPP_MOV(__float_as_uint(v), 0x130)); }   // wave_shl:1

// maximum over the wave, result in every lane
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
  v = max(v, OBF_DPP_MOV(v, 0xB1));
  v = max(v, OBF_DPP_MOV(v, 0x4E));
  v = max(v, OBF_DPP_MOV(v, 0x141));
  v = max(v, OBF_DPP_MOV(v, 0x140));
  const auto a = __builtin_amdgcn_permlane16_swap(v, v, false, false);     // rows 0/1 and 2/3 meet
  v = max((uint32_t)a[0], (uint32_t)a[1]);
  const auto b = __builtin_amdgcn_permlane32_swap(v, v, false, false);     // the two halves meet
  return max((uint32_t)b[0], (uint32_t)b[1]);
}

__device__ __forceinline__ uint64_t obf_dpp_mov64(uint64_t v, int which) {
  uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
  switch (which) {
    case 0: lo = OBF_DPP_MOV(lo, 0xB1); hi = OBF_DPP_MOV(hi, 0xB1); break;
    case 1: lo = OBF_DPP_MOV(lo, 0x4E); hi = OBF_DPP_MOV(hi, 0x4E); break;
    case 2: lo = OBF_DPP_MOV(lo, 0x141); hi = OBF_DPP_MOV(hi, 0x141); break;
    default: lo = OBF_DPP_MOV(lo, 0x140); hi = OBF_DPP_MOV(hi, 0x140); break;
  }
  return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
#pragma unroll
  for (int k = 0; k < 4; ++k) { const uint64_t o = obf_dpp_mov64(v, k); v = o > v ? o : v; }
  {
    const auto lo = __builtin_amdgcn_permlane16_swap((uint32_t)v, (uint32_t)v, false, false);
    const auto hi = __builtin_amdgcn_permlane16_swap((uint32_t)(v >> 32), (uint32_t)(v >> 32), false, false);
    const uint64_t a = ((uint64_t)hi[0] << 32) | lo[0], b = ((uint64_t)hi[1] << 32) | lo[1];
    v = a > b ? a : b;
  }
  {
    const auto lo = __builtin_amdgcn_permlane32_swap((uint32_t)v, (uint32_t)v, false, false);
    const auto hi = __builtin_amdgcn_permlane32_swap((uint32_t)(v >> 32), (uint32_t)(v >> 32), false, false);
    const uint64_t a = ((uint64_t)hi[0] << 32) | lo[0], b = ((uint64_t)hi[1] << 32) | lo[1];
    v = a > b ? a : b;
  }
  return v;
}

// sum over each 16-lane row, result in every lane of the row (the same value in all of them)
__device__ __forceinline__ double row16_sum_f64(double v) {
#pragma unroll
  for (int k = 0; k < 4; ++k) v += __longlong_as_double((long long)obf_dpp_mov64((uint64_t)__double_as_longlong(v), k));
  return v;
}

// sum over each aligned group of 32 lanes (two rows), result in every lane of the group
__device__ __forceinline__ double row32_sum_f64(double v) {
  v = row16_sum_f64(v);
  const uint64_t u = (uint64_t)__double_as_longlong(v);
  const auto lo = __builtin_amdgcn_permlane16_swap((uint32_t)u, (uint32_t)u, false, false);
  const auto hi = __builtin_amdgcn_permlane16_swap((uint32_t)(u >> 32), (uint32_t)(u >> 32), false, false);
  const double a = __longlong_as_double((long long)(((uint64_t)hi[0] << 32) | lo[0]));   // rows 0, 0, 2, 2
  const double b = __longlong_as_double((long long)(((uint64_t)hi[1] << 32) | lo[1]));   // rows 1, 1, 3, 3
  return a + b;
}

}  // namespace obf
