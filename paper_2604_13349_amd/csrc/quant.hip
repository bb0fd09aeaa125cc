// Post-hoc int8 / int4 codes for relay rows (the "+ int8" rows of App. E's comparison table).  The paper names no
// scheme; the one taken here reproduces its ratios: every row carries its own asymmetric code and two half-precision
// numbers, zero = fp16(min x), scale = fp16((max x - min x) / L), L = 2^bits - 1, q = clamp(rint((x - zero) / scale), 0, L).
// The integer decision is taken in single precision with individually rounded subtract, divide and round-to-even.
#include <hip/hip_fp16.h>
#include "common.hpp"

namespace obf {

constexpr int QT_THREADS = 256;

// one wave per row; lane l owns columns l and l + 64
template <typename T>
__global__ __launch_bounds__(QT_THREADS) void k_quant_rows(const T* __restrict__ X, long n_rows, int d, int bits,
                                                           uint8_t* __restrict__ codes, uint16_t* __restrict__ scale,
                                                           uint16_t* __restrict__ zero) {
  const long row = (long)blockIdx.x * (QT_THREADS / 64) + (threadIdx.x >> 6);
  if (row >= n_rows) return;
  const int lane = threadIdx.x & 63;
  const T* x = X + row * d;
  const bool two = lane + 64 < d;
  const float a = Elem<T>::load(x + lane), b = two ? Elem<T>::load(x + lane + 64) : a;      // d is 64 or 128
  float lo = fminf(a, b), hi = fmaxf(a, b);
  for (int off = 32; off > 0; off >>= 1) { lo = fminf(lo, __shfl_xor(lo, off)); hi = fmaxf(hi, __shfl_xor(hi, off)); }
  const float L = (float)((1 << bits) - 1);
  const __half zh = __float2half_rn(lo), sh = __float2half_rn(__fdiv_rn(__fsub_rn(hi, lo), L));
  const float z = __half2float(zh), s = __half2float(sh);
  auto code = [&](float v) -> uint32_t {
    if (!(s > 0.f)) return 0u;
    const float q = rintf(__fdiv_rn(__fsub_rn(v, z), s));
    return (uint32_t)fminf(fmaxf(q, 0.f), L);
  };
  const uint32_t qa = code(a), qb = code(b);
  if (bits == 8) {
    codes[row * d + lane] = (uint8_t)qa;
    if (two) codes[row * d + lane + 64] = (uint8_t)qb;
  } else {
    // two codes per byte, the even column in the low half: lane pairs (2i, 2i + 1) meet
    const uint32_t na = __shfl_xor(qa, 1), nb = __shfl_xor(qb, 1);
    if ((lane & 1) == 0) {
      codes[row * (d / 2) + lane / 2] = (uint8_t)(qa | (na << 4));
      if (two) codes[row * (d / 2) + (lane + 64) / 2] = (uint8_t)(qb | (nb << 4));
    }
  }
  if (lane == 0) { scale[row] = __half_as_ushort(sh); zero[row] = __half_as_ushort(zh); }
}

template <typename T>
__global__ __launch_bounds__(QT_THREADS) void k_dequant_rows(const uint8_t* __restrict__ codes, const uint16_t* __restrict__ scale,
                                                             const uint16_t* __restrict__ zero, long n_rows, int d, int bits,
                                                             T* __restrict__ X) {
  const long e = (long)blockIdx.x * QT_THREADS + threadIdx.x;
  if (e >= n_rows * d) return;
  const long row = e / d;
  const int c = (int)(e - row * d);
  const uint32_t q = (bits == 8) ? codes[e] : ((codes[row * (d / 2) + c / 2] >> ((c & 1) * 4)) & 15u);
  const float s = __half2float(__ushort_as_half(scale[row])), z = __half2float(__ushort_as_half(zero[row]));
  Elem<T>::store(X + e, fmaf(s, (float)q, z));
}

obf_status_t launch_quant_rows(const void* X, long n_rows, int d, int dtype, int bits, uint8_t* codes, uint16_t* scale,
                               uint16_t* zero, hipStream_t st) {
  if (n_rows == 0) return OBF_OK;
  const unsigned grid = (unsigned)((n_rows + QT_THREADS / 64 - 1) / (QT_THREADS / 64));
  if (dtype == OBF_BF16) hipLaunchKernelGGL(k_quant_rows<uint16_t>, dim3(grid), dim3(QT_THREADS), 0, st, (const uint16_t*)X, n_rows, d, bits, codes, scale, zero);
  else hipLaunchKernelGGL(k_quant_rows<float>, dim3(grid), dim3(QT_THREADS), 0, st, (const float*)X, n_rows, d, bits, codes, scale, zero);
  return check_launch("quantize rows");
}

obf_status_t launch_dequant_rows(const uint8_t* codes, const uint16_t* scale, const uint16_t* zero, long n_rows, int d, int dtype,
                                 int bits, void* X, hipStream_t st) {
  if (n_rows == 0) return OBF_OK;
  const unsigned grid = (unsigned)((n_rows * d + QT_THREADS - 1) / QT_THREADS);
  if (dtype == OBF_BF16) hipLaunchKernelGGL(k_dequant_rows<uint16_t>, dim3(grid), dim3(QT_THREADS), 0, st, codes, scale, zero, n_rows, d, bits, (uint16_t*)X);
  else hipLaunchKernelGGL(k_dequant_rows<float>, dim3(grid), dim3(QT_THREADS), 0, st, codes, scale, zero, n_rows, d, bits, (float*)X);
  return check_launch("dequantize rows");
}

}  // namespace obf
