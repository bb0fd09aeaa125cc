// Fast decision "the retained values span all of R^d" (then Eq. 3's residual is identically zero and
// the head stays plain eviction) for bf16 caches with head_dim 128 and more retained rows than
// head_dim.  It is a sufficient test only: heads it cannot certify go to the reference-precision
// basis kernel.
//
//   G   = V_s^T V_s over a strided subset V_s of the retained rows (all rows up to 1536), on the matrix
//         cores: products of bf16 values are exact in fp32, accumulation is fp32;
//   mu  = (max(n, d) 2^-23)^2 ||V_keep||_F^2  +  allowance for the fp32 error of G and of the
//         factorisation;
//   if the Cholesky factorisation of G - mu I runs through with positive pivots, then
//   sigma_min(V_keep)^2 >= lambda_min(G) > (max(n, d) 2^-23)^2 sigma_max(V_keep)^2, i.e. every singular
//   value is above the rank rule's threshold: r = d.
#include "common.hpp"

namespace obf {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int KC_THREADS = 256;
constexpr int KC_D = 128;
constexpr int KC_TILE = 64;              // rows staged per iteration
constexpr int KC_LDT = 132;              // staging row stride in bf16 (264 bytes: the two lane halves, 8 rows apart, use different banks)
constexpr int KC_LDG = 129;              // Gram row stride in floats
constexpr int KC_MAXROWS = 1536;
constexpr float kCertErr = 4.0e-6f;      // allowance for fp32 Gram + Cholesky error, relative to trace(G)

union FragU { uint32_t w[4]; bf16x8 v; };

__global__ __launch_bounds__(KC_THREADS) void k_bf_keep_cert(const uint16_t* __restrict__ V,
                                                             const float* __restrict__ scores,
                                                             const int32_t* __restrict__ idx,
                                                             const int32_t* __restrict__ n_keep, int N, int max_budget,
                                                             int rank, HeadState* __restrict__ state,
                                                             int32_t* __restrict__ decided) {
  __shared__ float G[KC_D * KC_LDG];                 // also the staging tile during the Gram phase
  __shared__ double red[KC_THREADS / 64];
  __shared__ int s_fail;
  uint16_t* stage = (uint16_t*)G;                    // [KC_TILE][KC_LDT]
  const int head = blockIdx.x;
  const int n = n_keep[head];
  const int n_del = N - n;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) decided[head] = 0;
  if (!(rank > 0 && n > KC_D && n_del > 0)) return;
  const float* sc = scores + (size_t)head * N;
  const int32_t* id = idx + (size_t)head * max_budget;
  const uint16_t* Vh = V + (size_t)head * N * KC_D;

  const int stride = (n + KC_MAXROWS - 1) / KC_MAXROWS;
  const int rows = (n + stride - 1) / stride;

  f32x16 acc[4];
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;

  for (int r0 = 0; r0 < rows; r0 += KC_TILE) {
    __syncthreads();
    // stage 64 rows: thread -> (row, 8-byte piece); 64 rows * 32 pieces = 2048 pieces
    for (int e = tid; e < KC_TILE * 32; e += KC_THREADS) {
      const int r = e >> 5, c = e & 31;
      uint2 val = make_uint2(0u, 0u);
      if (r0 + r < rows) val = *(const uint2*)(Vh + (size_t)id[(size_t)(r0 + r) * stride] * KC_D + c * 4);
      *(uint2*)(stage + r * KC_LDT + c * 4) = val;
    }
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < KC_TILE / 16; ++ks) {
      FragU f[4];
      const int tb = ks * 16 + (lane >> 5) * 8;
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        const uint16_t* p = stage + tb * KC_LDT + cb * 32 + (lane & 31);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const uint32_t lo = p[(2 * i) * KC_LDT], hi = p[(2 * i + 1) * KC_LDT];
          f[cb].w[i] = lo | (hi << 16);
        }
      }
      // wave w owns output rows (channels) w*32..w*32+31 and all four column blocks
      FragU own = f[0];
      if (wave == 1) own = f[1];
      if (wave == 2) own = f[2];
      if (wave == 3) own = f[3];
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(own.v, f[cb].v, acc[cb], 0, 0, 0);
    }
  }
  __syncthreads();
#pragma unroll
  for (int cb = 0; cb < 4; ++cb)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int row = wave * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
      const int col = cb * 32 + (lane & 31);
      G[row * KC_LDG + col] = acc[cb][i];
    }
  __syncthreads();

  // trace(G) and ||V_keep||_F^2 (equal when every retained row entered G)
  double part = 0.0;
  if (tid < KC_D) part = (double)G[tid * KC_LDG + tid];
  for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off);
  if (lane == 0) red[wave] = part;
  __syncthreads();
  const double tr = (red[0] + red[1]) + (red[2] + red[3]);
  __syncthreads();
  double f2 = tr;
  if (stride > 1) {
    // squared norms of all retained rows: 16 lanes per row, 8 bf16 each
    double p2 = 0.0;
    const int sub = tid >> 4, piece = tid & 15;
    for (int r = sub; r < n; r += KC_THREADS / 16) {
      const uint4 q = *(const uint4*)(Vh + (size_t)id[r] * KC_D + piece * 8);
      const uint32_t w4[4] = {q.x, q.y, q.z, q.w};
      float s = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float a = __uint_as_float(w4[i] << 16), b = __uint_as_float(w4[i] & 0xffff0000u);
        s = fmaf(a, a, s); s = fmaf(b, b, s);
      }
      p2 += (double)s;
    }
    for (int off = 32; off > 0; off >>= 1) p2 += __shfl_xor(p2, off);
    if (lane == 0) red[wave] = p2;
    __syncthreads();
    f2 = (red[0] + red[1]) + (red[2] + red[3]);
    __syncthreads();
  }
  const double thr_rel = (double)max(n, KC_D) * 1.1920928955078125e-07;
  const float mu = (float)(thr_rel * thr_rel * f2 + (double)kCertErr * tr);

  // right-looking Cholesky of G - mu I on the lower triangle; any non-positive pivot -> not certified
  if (tid == 0) s_fail = 0;
  if (tid < KC_D) G[tid * KC_LDG + tid] -= mu;
  __syncthreads();
  const int ty = tid >> 4, tx = tid & 15;
  for (int k = 0; k < KC_D; ++k) {
    const float piv = G[k * KC_LDG + k];
    if (!(piv > 0.f)) { if (tid == 0) s_fail = 1; break; }           // uniform: every thread reads the same pivot
    const float rinv = rsqrtf(piv);
    __syncthreads();
    for (int i = k + 1 + tid; i < KC_D; i += KC_THREADS) G[i * KC_LDG + k] *= rinv;
    __syncthreads();
    // trailing update on 16 x 16 interleaved blocks: rows i = ty + 16a, cols j = tx + 16b, k < j <= i
    for (int i = ty + ((k + 1 - ty + 15) >> 4) * 16; i < KC_D; i += 16) {
      const float lik = G[i * KC_LDG + k];
      for (int j = tx + ((k + 1 - tx + 15) >> 4) * 16; j <= i; j += 16) G[i * KC_LDG + j] -= lik * G[j * KC_LDG + k];
    }
    __syncthreads();
  }
  __syncthreads();
  if (s_fail) return;

  // certified: r = d, OBF is the identity on this head; fill in the demand sums (Eq. 6) for the diagnostics
  double pk = 0.0, pt = 0.0;
  for (int i = tid; i < n; i += KC_THREADS) pk += (double)sc[id[i]];
  for (int i = tid; i < N; i += KC_THREADS) pt += (double)sc[i];
  for (int off = 32; off > 0; off >>= 1) { pk += __shfl_xor(pk, off); pt += __shfl_xor(pt, off); }
  __shared__ double red2[KC_THREADS / 64];
  if (lane == 0) { red[wave] = pk; red2[wave] = pt; }
  __syncthreads();
  if (tid == 0) {
    const double a_keep = ((red[0] + red[1]) + red[2]) + red[3];
    const double a_tot = ((red2[0] + red2[1]) + red2[2]) + red2[3];
    HeadState s;
    s.a_keep = a_keep; s.a_del = fmax(a_tot - a_keep, 0.0); s.n_keep = n; s.n_del = n_del; s.r_keep = KC_D; s.active = 0;
    s.k_used = 0; s.pad = 0; s.rcr = 0.f; s.ivn = 0.f;
    state[head] = s;
    decided[head] = 1;
  }
}

bool keep_cert_supported(const Dims& m) { return m.dtype == OBF_BF16 && m.d == KC_D; }

obf_status_t launch_keep_cert(const Dims& m, const void* V, const float* scores, const int32_t* idx,
                              const int32_t* n_keep, int32_t max_budget, int32_t rank, HeadState* state,
                              int32_t* decided, hipStream_t st) {
  { ProfScope prof_(ST_KEEP_CERT, st);
    hipLaunchKernelGGL(k_bf_keep_cert, dim3(m.heads), dim3(KC_THREADS), 0, st, (const uint16_t*)V, scores, idx, n_keep,
                       m.N, max_budget, rank, state, decided); }
  return check_launch("backfill keep_cert");
}

}  // namespace obf
