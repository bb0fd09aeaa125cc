// Retained-span basis (Eq. 2) for heads with at most head_dim retained rows: the budget is below the
// head dimension, so the span always leaves a complement and Orthogonal BackFill (Sec. 4.4) is active.
//
// Per head (one workgroup of 16 x 32 threads), everything in double precision:
//   C = A A^T, the n x n Gram matrix of the retained rows A (entries of A are exact in float; products and
//       sums are taken in double), kept in registers (thread (ty, tx) owns C[ty + 16a][tx + 32b]; a single-precision
//       copy in LDS serves the power iteration only);
//   sigma_max^2 = lambda_max(C) by power iteration (the rank rule's threshold);
//   pivoted Gram-Schmidt on the rows of A, which live in registers (thread (ty, tx) owns A[ty + 16a][tx*CW ..]):
//       the pivot is the row with the largest remaining squared norm, read off the diagonal of C; the
//       projection coefficients of all rows onto the new direction are row j of C over sqrt(C[j][j]), so a
//       step is one rank-1 update of C and one of A, both in registers (no inner products; the owners of row j publish
//       it, two barriers);
//   rows whose remaining norm is at or below sigma_max * max(n, d) * 2^-23 end the loop: r = number of steps.
// Row s of the basis is written as soon as it is final.
#include "common.hpp"
#include "wave_ops.hpp"

namespace obf {

constexpr int KS_THREADS = 512;
constexpr int KS_WAVES = KS_THREADS / 64;
constexpr double kRankEpsKs = 1.1920928955078125e-07;   // 2^-23, the rank rule's epsilon

__device__ __forceinline__ double ks_block_sum(double v, double* red /*[KS_WAVES]*/) {
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  double s = 0.0;
  for (int i = 0; i < KS_WAVES; ++i) s += red[i];
  return s;
}

template <typename T, int CW> struct RowLoad;
template <> struct RowLoad<uint16_t, 2> {
  static __device__ __forceinline__ void get(const uint16_t* p, double (&o)[2]) {
    const uint32_t w = *(const uint32_t*)p;
    o[0] = (double)__uint_as_float(w << 16); o[1] = (double)__uint_as_float(w & 0xffff0000u);
  }
};
template <> struct RowLoad<uint16_t, 4> {
  static __device__ __forceinline__ void get(const uint16_t* p, double (&o)[4]) {
    const uint2 q = *(const uint2*)p;
    const uint32_t w[2] = {q.x, q.y};
#pragma unroll
    for (int i = 0; i < 2; ++i) { o[2 * i] = (double)__uint_as_float(w[i] << 16); o[2 * i + 1] = (double)__uint_as_float(w[i] & 0xffff0000u); }
  }
};
template <> struct RowLoad<float, 4> {
  static __device__ __forceinline__ void get(const float* p, double (&o)[4]) {
    const float4 q = *(const float4*)p;
    o[0] = (double)q.x; o[1] = (double)q.y; o[2] = (double)q.z; o[3] = (double)q.w;
  }
};
template <> struct RowLoad<float, 2> {
  static __device__ __forceinline__ void get(const float* p, double (&o)[2]) {
    const float2 q = *(const float2*)p;
    o[0] = (double)q.x; o[1] = (double)q.y;
  }
};

struct KsShared {
  double red[KS_WAVES];
  float xv[128], yp[4][128];         // power iteration: iterate, partial products
  double qrow[128];                  // row j of A at a step (unscaled)
  double crow[128];                  // row j of C at a step (before the loop: the diagonal of C)
  uint32_t wkey[2][2];
};

// Stages 16-byte pieces of the retained rows into LDS as float, row stride d + 1.
template <typename T, int D>
__device__ __forceinline__ void ks_stage_rows(const T* __restrict__ Vh, const int32_t* __restrict__ id, int n, float* stg) {
  constexpr int EPP = 16 / (int)sizeof(T);                     // elements per piece
  constexpr int PPR = D / EPP;                                 // pieces per row
  for (int e = threadIdx.x; e < n * PPR; e += KS_THREADS) {
    const int i = e / PPR, pc = e - i * PPR;
    const uint4 q = *(const uint4*)(Vh + (size_t)id[i] * D + pc * EPP);
    float* o = stg + i * (D + 1) + pc * EPP;
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
    if constexpr (sizeof(T) == 2) {
#pragma unroll
      for (int k = 0; k < 4; ++k) { o[2 * k] = __uint_as_float(w[k] << 16); o[2 * k + 1] = __uint_as_float(w[k] & 0xffff0000u); }
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k) o[k] = __uint_as_float(w[k]);
    }
  }
}

// One head.  TI = ceil(n / 16) rounded up to even, CW = d / 32.  Returns r.
// C is stored padded to NP = 16 TI rows and columns (zero beyond n), so that every index below is an immediate.
template <typename T, int TI, int CW>
__device__ __forceinline__ int ks_head(const T* __restrict__ Vh, const int32_t* __restrict__ id, int n, float* __restrict__ bh,
                       double* C, KsShared& sh) {
  constexpr int d = 32 * CW;
  constexpr int TJ = TI / 2;                                   // column blocks of 32 of a thread's C elements
  constexpr int NP = 16 * TI;
  const int tid = threadIdx.x, lane = tid & 63;
  const int ty = tid >> 5, tx = tid & 31;
  float* stg = (float*)C;                                      // Gram staging [n][d + 1], before the copy of C is stored
  float* Cf = (float*)C;                                       // [NP][NP]

  // ---- Gram matrix: thread (ty, tx) accumulates C[ty + 16a][tx + 32b]
  double creg[TI][TJ];
  {
#pragma unroll
    for (int a = 0; a < TI; ++a)
#pragma unroll
      for (int b = 0; b < TJ; ++b) creg[a][b] = 0.0;
    __syncthreads();
    ks_stage_rows<T, d>(Vh, id, n, stg);
    __syncthreads();
    const float* ap[TI];
    const float* bp[TJ];
#pragma unroll
    for (int a = 0; a < TI; ++a) ap[a] = stg + min(ty + 16 * a, n - 1) * (d + 1);
#pragma unroll
    for (int b = 0; b < TJ; ++b) bp[b] = stg + min(tx + 32 * b, n - 1) * (d + 1);
#pragma unroll 4
    for (int c = 0; c < d; ++c) {
      double av[TI], bv[TJ];
#pragma unroll
      for (int a = 0; a < TI; ++a) av[a] = (double)ap[a][c];
#pragma unroll
      for (int b = 0; b < TJ; ++b) bv[b] = (double)bp[b][c];
#pragma unroll
      for (int a = 0; a < TI; ++a)
#pragma unroll
        for (int b = 0; b < TJ; ++b) creg[a][b] = fma(av[a], bv[b], creg[a][b]);
    }
    __syncthreads();                                           // the staging area aliases C
#pragma unroll
    for (int a = 0; a < TI; ++a)
#pragma unroll
      for (int b = 0; b < TJ; ++b) {
        const int i = ty + 16 * a, jj = tx + 32 * b;
        if (!(i < n && jj < n)) creg[a][b] = 0.0;                // rows past n were clamped reads
        Cf[i * NP + jj] = (float)creg[a][b];                     // single-precision copy for the power iteration
        if (i == jj) sh.crow[i] = creg[a][b];
      }
    __syncthreads();
  }

  // ---- sigma_max^2 = lambda_max(C): power iteration in single precision (the estimate only sets the rank rule's
  // threshold, where a percent is immaterial).  Each quarter of the workgroup (a wave pair) takes every fourth row of
  // C for all columns, the partial products meet in LDS.  The iterate is scaled by the first step's estimate only;
  // the last step takes the true ratio.
  if (tid < 128) sh.xv[tid] = (tid < n) ? (float)(1.0 / sqrt((double)n)) * (1.f + 0.01f * (float)(tid % 7)) : 0.f;
  __syncthreads();
  double lam = 0.0;
  float scale = 1.f;
  const int prow = tid & 127, ppart = tid >> 7;                // ppart is uniform over a wave
  const bool pact = prow < NP;
  const float* cp = Cf + ppart * NP + (pact ? prow : 0);       // C symmetric: column reads are row reads
  const float* xp = sh.xv + ppart;
  constexpr int kPowerIters = 12;
  for (int it = 0; it < kPowerIters; ++it) {
    float y0 = 0.f, y1 = 0.f;
#pragma unroll
    for (int u = 0; u < NP / 4; u += 2) {
      y0 = fmaf(cp[(4 * u) * NP], xp[4 * u], y0);
      y1 = fmaf(cp[(4 * u + 4) * NP], xp[4 * u + 4], y1);
    }
    sh.yp[ppart][prow] = pact ? y0 + y1 : 0.f;
    lds_barrier();
    float y = 0.f;
    if (tid < 128) y = (sh.yp[0][tid] + sh.yp[1][tid]) + (sh.yp[2][tid] + sh.yp[3][tid]);
    if (it == 0 || it == kPowerIters - 1) {
      const float x0 = (tid < 128) ? sh.xv[tid] : 0.f;
      const double n2 = ks_block_sum((double)y * y, sh.red);
      const double d2 = ks_block_sum((double)x0 * x0, sh.red);
      lam = sqrt(n2 / fmax(d2, 1e-300));
      if (!(lam > 0.0)) break;
      scale = (float)(1.0 / lam);
    }
    if (tid < 128) sh.xv[tid] = y * scale;
    lds_barrier();
  }
  const double thr = sqrt(lam) * (double)max(n, d) * kRankEpsKs;
  const double thr2 = thr * thr;                               // pivots are squared distances

  // ---- rows of A: thread (ty, tx) owns A[ty + 16a][tx*CW ..]
  double areg[TI][CW];
  {
    int rid[TI];
#pragma unroll
    for (int a = 0; a < TI; ++a) rid[a] = id[min(ty + 16 * a, n - 1)];
#pragma unroll
    for (int a = 0; a < TI; ++a) RowLoad<T, CW>::get(Vh + (size_t)rid[a] * d + tx * CW, areg[a]);
#pragma unroll
    for (int a = 0; a < TI; ++a)
      if (ty + 16 * a >= n) {
#pragma unroll
        for (int c = 0; c < CW; ++c) areg[a][c] = 0.0;
      }
  }

  // ---- pivoted Gram-Schmidt driven by C
  double dg = (tid < n) ? sh.crow[tid] : -1.0;                 // threads < n: remaining squared norm of row tid
  bool used = false;
  // Pivot search key: the high word of the (positive) double, low 7 bits replaced by 127 - row, so that the
  // maximum over the keys is the largest remaining norm (to 13 mantissa bits), lowest row first among equals.
  auto publish = [&](int buf) {
    if (tid < 128) {
      uint32_t key = (!used && dg > 0.0) ? ((((uint32_t)(((uint64_t)__double_as_longlong(dg)) >> 32)) & ~0x7Fu) | (uint32_t)(127 - tid)) : 0u;
      key = wave_max_u32(key);
      if (lane == 0) sh.wkey[buf][tid >> 6] = key;
    }
  };
  publish(0);
  __syncthreads();
  int r = 0;
  for (int s = 0; s < n; ++s) {
    const uint32_t key = max(sh.wkey[s & 1][0], sh.wkey[s & 1][1]);
    if (key == 0u) break;
    const int j = 127 - (int)(key & 0x7Fu);
    if (ty == (j & 15)) {                                      // row j of C and of A sit in these threads, register j / 16
      double* qr = sh.qrow + tx * CW;
      double* cr = sh.crow + tx;
#define KS_ROW(k) case k: if constexpr (k < TI) { \
        _Pragma("unroll") for (int c = 0; c < CW; ++c) qr[c] = areg[k][c]; \
        _Pragma("unroll") for (int b = 0; b < TJ; ++b) cr[32 * b] = creg[k][b]; } break;
      switch (j >> 4) { KS_ROW(0) KS_ROW(1) KS_ROW(2) KS_ROW(3) KS_ROW(4) KS_ROW(5) KS_ROW(6) KS_ROW(7) default: break; }
#undef KS_ROW
    }
    lds_barrier();
    const double xjj = sh.crow[j];
    if (!(xjj > thr2)) break;                                  // the largest remaining norm is at the rank threshold (uniform)
    const double inv = rsqrt(xjj);                             // 1 / remaining norm of row j
    double la[TI];
#pragma unroll
    for (int a = 0; a < TI; ++a) la[a] = sh.crow[ty + 16 * a] * inv;     // <row, new direction>
    {
      double q[CW];
#pragma unroll
      for (int c = 0; c < CW; ++c) q[c] = sh.qrow[tx * CW + c] * inv;    // the new direction
#pragma unroll
      for (int a = 0; a < TI; ++a)
#pragma unroll
        for (int c = 0; c < CW; ++c) areg[a][c] = fma(-la[a], q[c], areg[a][c]);
      if (ty == 0) {
        float* o = bh + (size_t)s * d + tx * CW;
        if constexpr (CW == 4) *(float4*)o = make_float4((float)q[0], (float)q[1], (float)q[2], (float)q[3]);
        else *(float2*)o = make_float2((float)q[0], (float)q[1]);
      }
    }
#pragma unroll
    for (int b = 0; b < TJ; ++b) {
      const double lbs = sh.crow[tx + 32 * b] * inv;
#pragma unroll
      for (int a = 0; a < TI; ++a) creg[a][b] = fma(-la[a], lbs, creg[a][b]);
    }
    if (tid < 128) {
      const double l = sh.crow[min(tid, NP - 1)] * inv;        // this thread's own row's coefficient
      if (tid == j) used = true;
      if (!used) dg -= l * l;
    }
    publish((s + 1) & 1);
    lds_barrier();
    r = s + 1;
  }
  __syncthreads();
  return r;
}

template <typename T, bool BIG>
__global__ __launch_bounds__(KS_THREADS, BIG ? 2 : 4) void k_bf_keep_basis_small(const T* __restrict__ V, const float* __restrict__ scores,
                                                                    const int32_t* __restrict__ idx,
                                                                    const int32_t* __restrict__ n_keep, int N, int d,
                                                                    int max_budget, int rank, HeadState* __restrict__ state,
                                                                    float* __restrict__ basis, int scs, int kvs) {
  const int head = blockIdx.x;
  const int n = n_keep[head];
  if (n > d) return;                         // heads of the general kernel
  if ((n > 96) != BIG) return;               // n > 96: larger LDS buffer and register budget, a launch of its own
  extern __shared__ double Cs[];             // staging area of the Gram accumulation, then the single-precision copy of C
  __shared__ KsShared sh;
  const int n_del = N - n;
  const float* sc = scores + (size_t)head * scs;
  const int32_t* id = idx + (size_t)head * max_budget;
  const T* Vh = V + (size_t)head * kvs * d;
  const int tid = threadIdx.x;

  // demand sums of Eq. 6, in double, fixed summation order
  double pk = 0.0, pt = 0.0;
  for (int i = tid; i < n; i += KS_THREADS) pk += (double)sc[id[i]];
  for (int i = tid; i < N; i += KS_THREADS) pt += (double)sc[i];
  const double a_keep = ks_block_sum(pk, sh.red);
  const double a_tot = ks_block_sum(pt, sh.red);
  double a_del = a_tot - a_keep;
  if (a_del < 0.0) a_del = 0.0;

  int r_keep = 0, active = 0;
  if (rank > 0 && n > 0 && n_del > 0) {
    float* bh = basis + (size_t)head * d * d;
    if constexpr (BIG) {
      r_keep = ks_head<T, 8, 4>(Vh, id, n, bh, Cs, sh);        // n > 96 implies d = 128
    } else if (d == 128) {
      if (n <= 32) r_keep = ks_head<T, 2, 4>(Vh, id, n, bh, Cs, sh);
      else if (n <= 64) r_keep = ks_head<T, 4, 4>(Vh, id, n, bh, Cs, sh);
      else r_keep = ks_head<T, 6, 4>(Vh, id, n, bh, Cs, sh);
    } else {
      if (n <= 32) r_keep = ks_head<T, 2, 2>(Vh, id, n, bh, Cs, sh);
      else r_keep = ks_head<T, 4, 2>(Vh, id, n, bh, Cs, sh);
    }
    active = (r_keep < d) ? 1 : 0;
  }
  if (tid == 0) {
    HeadState s;
    s.a_keep = a_keep; s.a_del = a_del; s.n_keep = n; s.n_del = n_del; s.r_keep = r_keep; s.active = active;
    s.k_used = 0; s.pad = 0; s.rcr = 0.f; s.ivn = 0.f;
    state[head] = s;
  }
}

// dynamic LDS of a launch whose heads keep at most nmax rows: the padded Gram matrix or the row staging
static size_t ks_smem(size_t nmax, int d) {
  const size_t np = (nmax + 31) / 32 * 32;
  return max(np * np * sizeof(float), nmax * (size_t)(d + 1) * sizeof(float));
}

template <typename T>
static obf_status_t run_small(const Dims& m, const void* V, const float* scores, const int32_t* idx,
                              const int32_t* n_keep, int32_t max_budget, int32_t rank, HeadState* state, float* basis,
                              hipStream_t st) {
  static std::mutex attr_mu;
  static uint64_t attr_seen = 0;
  once_per_device(attr_mu, attr_seen, [] {
    (void)hipFuncSetAttribute((const void*)k_bf_keep_basis_small<T, false>, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 129 * 4);
    (void)hipFuncSetAttribute((const void*)k_bf_keep_basis_small<T, true>, hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 129 * 4);
  });
  const size_t nmax = (size_t)min(max_budget, m.d);
  hipLaunchKernelGGL((k_bf_keep_basis_small<T, false>), dim3(m.heads), dim3(KS_THREADS), ks_smem(min(nmax, (size_t)96), m.d), st,
                     (const T*)V, scores, idx, n_keep, m.N, m.d, max_budget, rank, state, basis, m.scs, m.kvs);
  if (check_launch("backfill keep_basis_small") != OBF_OK) return OBF_ERR_HIP;
  if (nmax > 96) {
    hipLaunchKernelGGL((k_bf_keep_basis_small<T, true>), dim3(m.heads), dim3(KS_THREADS), ks_smem(nmax, m.d), st,
                       (const T*)V, scores, idx, n_keep, m.N, m.d, max_budget, rank, state, basis, m.scs, m.kvs);
    if (check_launch("backfill keep_basis_small (wide)") != OBF_OK) return OBF_ERR_HIP;
  }
  return OBF_OK;
}

obf_status_t launch_keep_basis_small(const Dims& m, const void* V, const float* scores, const int32_t* idx,
                                     const int32_t* n_keep, int32_t max_budget, int32_t rank, HeadState* state,
                                     float* basis, hipStream_t st) {
  if (m.dtype == OBF_BF16) return run_small<uint16_t>(m, V, scores, idx, n_keep, max_budget, rank, state, basis, st);
  return run_small<float>(m, V, scores, idx, n_keep, max_budget, rank, state, basis, st);
}

}  // namespace obf
