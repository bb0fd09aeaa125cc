// Orthogonal BackFill (Sec. 4.4, Eq. 2-7; Alg. 3) on one GPU.
//
//   keep_basis : per head, demand sums (Eq. 6), dimension r and an orthonormal basis Q of the span of
//                the retained values (Eq. 2).  r == d means the orthogonal complement is {0}: the
//                residual of Eq. 3 vanishes identically and the head is left as plain eviction.
//                Three kernels share the heads: the full-rank certificate (keep_cert.hip, n > d), the
//                small-budget kernel (keep_basis_small.hip, n <= d) and k_bf_keep_basis below (n > d, not
//                certified).
//   del_stats  : for heads that still need it, one streaming pass over V accumulating the Gram
//                matrix V_del^T V_del, the mass-weighted sum of deleted values and ||V_del||_F^2
//                (del_stats_mfma.hip for bf16 head_dim-128 caches, k_bf_del_stats below otherwise).
//                R itself (Eq. 3) is never materialised: R^T R = P (V_del^T V_del) P and
//                sum_j w_j R_j = P sum_j w_j V_j with P = I - Q Q^T.
//   finalize   : per head, an orthonormal basis Z of the complement of the retained span, the eigenpairs of
//                Z G Z^T (those of P G P, i.e. the top right singular vectors of R; App. H: same subspace as
//                the SVD of R), rbar (Eq. 4), Delta (Eq. 5), delta (Eq. 6), and V* = V_keep + delta on every
//                retained row (Eq. 7), rounded once to the I/O dtype.
// The basis kernels may run on a second stream beside the gather and the statistics pass (small budgets).
#include "common.hpp"
#include "wave_ops.hpp"
#include "tri_eigs.hpp"

namespace obf {

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int KB_THREADS = 256;
constexpr int KB_WAVES = KB_THREADS / 64;
constexpr double kRankEps = 1.1920928955078125e-07;   // 2^-23, the rank rule's epsilon
constexpr float kRcrSkip = 1.0e-6f;                   // "||R||_F negligible": ||R||^2 <= 1e-6 ||V_del||^2
constexpr float kEigFloor = 1.0e-6f;                  // resolution of the fp32 residual Gram (relative)

// ------------------------------------------------------------------------------------------------
// small block helpers (KB_THREADS threads)
__device__ __forceinline__ double wave_sum(double v) {
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

__device__ __forceinline__ double block_sum(double v, double* red /*[KB_WAVES]*/) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  double s = 0.0;
  for (int i = 0; i < KB_WAVES; ++i) s += red[i];
  return s;
}

// Pivoted modified Gram-Schmidt on the m rows (dimension d) of W in LDS, double precision.
// Rows are orthonormalised in place in pivot order; returns the number of rows whose remaining
// norm exceeded thr_abs.  rows 0..r-1 of W are the basis on exit.
__device__ int pivoted_mgs(double* W, int m, int d, double thr_abs, double* red, int* ired) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __shared__ double nrm2[128];
  int r = 0;
  for (int k = 0; k < m; ++k) {
    // remaining squared norms, recomputed every step (no downdating drift)
    for (int i = k + wave; i < m; i += KB_WAVES) {
      double s = 0.0;
      for (int c = lane; c < d; c += 64) { const double x = W[i * d + c]; s += x * x; }
      s = wave_sum(s);
      if (lane == 0) nrm2[i] = s;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      int p = k; double best = nrm2[k];
      for (int i = k + 1; i < m; ++i) if (nrm2[i] > best) { best = nrm2[i]; p = i; }   // first maximum
      ired[0] = p; red[0] = best;
    }
    __syncthreads();
    const int p = ired[0];
    const double best = red[0];
    if (!(sqrt(best) > thr_abs)) break;
    const double inv = 1.0 / sqrt(best);
    // swap rows p and k, normalise row k
    for (int c = threadIdx.x; c < d; c += KB_THREADS) {
      const double a = W[p * d + c], b = W[k * d + c];
      W[p * d + c] = b; W[k * d + c] = a * inv;
    }
    __syncthreads();
    // remove the new direction from the remaining rows (twice: keeps orthogonality at double precision)
    for (int pass = 0; pass < 2; ++pass) {
      for (int i = k + 1 + wave; i < m; i += KB_WAVES) {
        double s = 0.0;
        for (int c = lane; c < d; c += 64) s += W[i * d + c] * W[k * d + c];
        s = wave_sum(s);
        for (int c = lane; c < d; c += 64) W[i * d + c] -= s * W[k * d + c];
      }
      __syncthreads();
    }
    r = k + 1;
  }
  __syncthreads();
  return r;
}

// Largest singular value of the m x d matrix W (LDS, double) by power iteration on W^T W.
__device__ double sigma_max_est(const double* W, int m, int d, double* x /*[d]*/, double* y /*[m]*/, double* red) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int c = threadIdx.x; c < d; c += KB_THREADS) x[c] = 1.0 / sqrt((double)d) * (1.0 + 0.01 * (c % 7));
  __syncthreads();
  double lam = 0.0;
  for (int it = 0; it < 24; ++it) {
    for (int i = wave; i < m; i += KB_WAVES) {
      double s = 0.0;
      for (int c = lane; c < d; c += 64) s += W[i * d + c] * x[c];
      s = wave_sum(s);
      if (lane == 0) y[i] = s;
    }
    __syncthreads();
    double part = 0.0;
    for (int c = threadIdx.x; c < d; c += KB_THREADS) {
      double s = 0.0;
      for (int i = 0; i < m; ++i) s += W[i * d + c] * y[i];
      x[c] = s;
      part += s * s;
    }
    const double n2 = block_sum(part, red);     // ||W^T W x||^2 with ||x|| = 1
    lam = sqrt(n2);                             // -> lambda_max(W^T W)
    if (!(lam > 0.0)) break;
    const double inv = 1.0 / lam;
    for (int c = threadIdx.x; c < d; c += KB_THREADS) x[c] *= inv;
    __syncthreads();
  }
  return sqrt(lam);
}

// Gram matrix V_keep^T V_keep (d x d, double) of the n retained rows into W (LDS, [d][d]); W doubles as the
// staging area while the sums are in registers.  16 x 16 threads, BS x BS outputs each (d = 16 BS): thread (ty, tx) owns G[ty + 16a][tx + 16b].
template <typename T, int BS>
__device__ void gram_rows_f64(const T* __restrict__ Vh, const int32_t* __restrict__ id, int n, double* W) {
  constexpr int D = 16 * BS;
  constexpr int EPP = 16 / (int)sizeof(T);                     // elements per 16-byte piece
  constexpr int PPR = D / EPP;                                 // pieces per row
  constexpr int TR = KB_THREADS / PPR;                         // rows staged per step
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  double acc[BS][BS];
#pragma unroll
  for (int a = 0; a < BS; ++a)
#pragma unroll
    for (int b = 0; b < BS; ++b) acc[a][b] = 0.0;
  float* rowbuf = (float*)W;                                   // [2][TR][D + 1]
  const int pr = threadIdx.x / PPR, pc = threadIdx.x - pr * PPR;
  auto fetch = [&](int i0) -> uint4 {
    const int i = i0 + pr;
    return (i < n) ? *(const uint4*)(Vh + (size_t)id[i] * D + pc * EPP) : make_uint4(0u, 0u, 0u, 0u);
  };
  auto put = [&](const uint4 q, int buf) {
    float* o = rowbuf + (buf * TR + pr) * (D + 1) + pc * EPP;
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
    if constexpr (sizeof(T) == 2) {
#pragma unroll
      for (int k = 0; k < 4; ++k) { o[2 * k] = __uint_as_float(w[k] << 16); o[2 * k + 1] = __uint_as_float(w[k] & 0xffff0000u); }
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k) o[k] = __uint_as_float(w[k]);
    }
  };
  uint4 nxt = fetch(0);
  int buf = 0;
  for (int i0 = 0; i0 < n; i0 += TR) {
    put(nxt, buf);
    nxt = fetch(i0 + TR);                                      // next rows are in flight during this step's sums
    __syncthreads();
    const float* rb = rowbuf + buf * TR * (D + 1);
#pragma unroll 2
    for (int i = 0; i < TR; ++i) {
      double av[BS], bv[BS];
#pragma unroll
      for (int a = 0; a < BS; ++a) av[a] = (double)rb[i * (D + 1) + ty + 16 * a];
#pragma unroll
      for (int b = 0; b < BS; ++b) bv[b] = (double)rb[i * (D + 1) + tx + 16 * b];
#pragma unroll
      for (int a = 0; a < BS; ++a)
#pragma unroll
        for (int b = 0; b < BS; ++b) acc[a][b] = fma(av[a], bv[b], acc[a][b]);
    }
    buf ^= 1;
  }
  __syncthreads();
#pragma unroll
  for (int a = 0; a < BS; ++a)
#pragma unroll
    for (int b = 0; b < BS; ++b) W[(ty + 16 * a) * D + tx + 16 * b] = acc[a][b];
  __syncthreads();
}

// True iff G - shift I (G symmetric d x d in LDS, d = 16 BS, left untouched) is positive definite: LDL^T without
// pivoting on a register copy, thread (ty, tx) of the 16 x 16 grid holding G[ty + 16a][tx + 16b].  Step k: the sixteen
// owners of row k publish it (two row buffers alternate, so one barrier per step), every thread divides by the pivot
// and updates its BS x BS entries.  Runs through iff every pivot is positive, i.e. iff lambda_min(G) > shift.
template <int BS>
__device__ bool shifted_ldl_positive(const double* W, double shift, double* row0, double* row1) {
  constexpr int D = 16 * BS;
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  double g[BS][BS];
#pragma unroll
  for (int a = 0; a < BS; ++a)
#pragma unroll
    for (int b = 0; b < BS; ++b) g[a][b] = W[(ty + 16 * a) * D + tx + 16 * b] - ((ty + 16 * a == tx + 16 * b) ? shift : 0.0);
  bool ok = true;
  for (int k = 0; k < D; ++k) {
    double* rb = (k & 1) ? row1 : row0;
    if ((k & 15) == ty) {
#pragma unroll
      for (int a = 0; a < BS; ++a)
        if (a == (k >> 4)) {
#pragma unroll
          for (int b = 0; b < BS; ++b) rb[tx + 16 * b] = g[a][b];
        }
    }
    __syncthreads();
    const double piv = rb[k];                                  // the same value in every thread
    if (!(piv > 0.0)) { ok = false; break; }
    const double ip = 1.0 / piv;
    double ri[BS], rj[BS];
#pragma unroll
    for (int a = 0; a < BS; ++a) ri[a] = rb[ty + 16 * a] * ip;
#pragma unroll
    for (int b = 0; b < BS; ++b) rj[b] = rb[tx + 16 * b];
#pragma unroll
    for (int a = 0; a < BS; ++a)
#pragma unroll
      for (int b = 0; b < BS; ++b) g[a][b] = fma(-ri[a], rj[b], g[a][b]);
  }
  __syncthreads();
  return ok;
}

// ------------------------------------------------------------------------------------------------
// Heads of the general basis kernel (more than d retained rows, not settled by the certificate), numbered in head
// order: the first kKeepGramSlots of them get their Gram matrix from partial matrices of kKeepGramChunks workgroups.
__device__ __forceinline__ bool kg_general(const int32_t* __restrict__ decided, const int32_t* __restrict__ n_keep, int h, int N,
                                           int d, int rank) {
  const int n = n_keep[h];
  return rank > 0 && n > d && N - n > 0 && !(decided && decided[h]);
}

// number of such heads below `head` (every thread gets it)
__device__ int kg_rank_of(const int32_t* __restrict__ decided, const int32_t* __restrict__ n_keep, int head, int N, int d, int rank,
                          double* red) {
  double c = 0.0;
  for (int h = threadIdx.x; h < head; h += KB_THREADS) c += kg_general(decided, n_keep, h, N, d, rank) ? 1.0 : 0.0;
  return (int)block_sum(c, red);
}

// the head whose number is `target`, or -1 (every thread gets it); s_i has KB_WAVES + 1 entries
__device__ int kg_head_of_rank(const int32_t* __restrict__ decided, const int32_t* __restrict__ n_keep, int heads, int N, int d,
                               int rank, int target, int* s_i) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (threadIdx.x == 0) s_i[KB_WAVES] = -1;
  int base = 0;
  for (int h0 = 0; h0 < heads; h0 += KB_THREADS) {
    const int h = h0 + threadIdx.x;
    const bool p = h < heads && kg_general(decided, n_keep, h, N, d, rank);
    const uint64_t mask = __ballot(p);
    __syncthreads();
    if (lane == 0) s_i[wave] = __popcll(mask);
    __syncthreads();
    int before = base, tot = 0;
    for (int w = 0; w < KB_WAVES; ++w) { if (w < wave) before += s_i[w]; tot += s_i[w]; }
    if (p && before + __popcll(mask & ((1ull << lane) - 1ull)) == target) s_i[KB_WAVES] = h;
    base += tot;
    if (base > target) break;                        // uniform: found
  }
  __syncthreads();
  return s_i[KB_WAVES];
}

// Partial Gram matrices: workgroup (c, s) sums chunk c of the retained rows of the s-th such head.
template <typename T>
__global__ __launch_bounds__(KB_THREADS) void k_bf_keep_gram_part(const T* __restrict__ V, const int32_t* __restrict__ idx,
                                                                  const int32_t* __restrict__ n_keep,
                                                                  const int32_t* __restrict__ decided, int heads, int N, int d,
                                                                  int max_budget, int rank, int kvs,
                                                                  double* __restrict__ gpart) {
  extern __shared__ double W[];
  __shared__ int s_i[KB_WAVES + 1];
  const int head = kg_head_of_rank(decided, n_keep, heads, N, d, rank, blockIdx.y, s_i);
  if (head < 0) return;
  const int n = n_keep[head];
  const int per = (n + kKeepGramChunks - 1) / kKeepGramChunks;
  const int i0 = min(n, (int)blockIdx.x * per), i1 = min(n, i0 + per);
  const int32_t* id = idx + (size_t)head * max_budget + i0;
  const T* Vh = V + (size_t)head * kvs * d;
  if (d == 128) gram_rows_f64<T, 8>(Vh, id, i1 - i0, W);
  else gram_rows_f64<T, 4>(Vh, id, i1 - i0, W);
  double* o = gpart + ((size_t)blockIdx.y * kKeepGramChunks + blockIdx.x) * d * d;
  for (int e = threadIdx.x; e < d * d; e += KB_THREADS) o[e] = W[e];
}

// ------------------------------------------------------------------------------------------------
// keep_basis
template <typename T>
__global__ __launch_bounds__(KB_THREADS) void k_bf_keep_basis(const T* __restrict__ V, const float* __restrict__ scores,
                                                              const int32_t* __restrict__ idx,
                                                              const int32_t* __restrict__ n_keep, int N, int d,
                                                              int max_budget, int rank, HeadState* __restrict__ state,
                                                              float* __restrict__ basis,
                                                              const int32_t* __restrict__ decided, int scs, int kvs,
                                                              const double* __restrict__ gpart /*nullable*/) {
  if (decided && decided[blockIdx.x]) return;        // settled by the fast full-rank test
  if (n_keep[blockIdx.x] <= d) return;               // heads of k_bf_keep_basis_small
  extern __shared__ double W[];            // [d][d] doubles (rows: vectors being orthonormalised / Gram)
  __shared__ double red[KB_WAVES];
  __shared__ int ired[2];
  __shared__ double xv[128], yv[128];
  __shared__ int perm[128];
  __shared__ uint64_t pkey[2];
  const int head = blockIdx.x;
  const int n = n_keep[head];
  const int n_del = N - n;
  const float* sc = scores + (size_t)head * scs;
  const int32_t* id = idx + (size_t)head * max_budget;
  const T* Vh = V + (size_t)head * kvs * d;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

  // demand sums of Eq. 6, in double, fixed summation order
  double pk = 0.0, pt = 0.0;
  for (int i = threadIdx.x; i < n; i += KB_THREADS) pk += (double)sc[id[i]];
  for (int i = threadIdx.x; i < N; i += KB_THREADS) pt += (double)sc[i];
  const double a_keep = block_sum(pk, red);
  const double a_tot = block_sum(pt, red);
  double a_del = a_tot - a_keep;
  if (a_del < 0.0) a_del = 0.0;

  int r_keep = 0, active = 0;
  if (rank > 0 && n > 0 && n_del > 0) {
    if (n <= d) {
      // rows of V_keep straight into LDS
      for (int e = threadIdx.x; e < n * d; e += KB_THREADS) {
        const int i = e / d, c = e - i * d;
        W[e] = (double)Elem<T>::load(Vh + (size_t)id[i] * d + c);
      }
      __syncthreads();
      const double smax = sigma_max_est(W, n, d, xv, yv, red);
      const double thr = smax * (double)max(n, d) * kRankEps;
      r_keep = pivoted_mgs(W, n, d, thr, red, ired);
    } else {
      // n > d: Gram matrix of the retained rows in double (inputs are exact, products exact),
      // diagonally pivoted Cholesky for the rank, then the rows of the factor span the row space.
      const int slot = gpart ? kg_rank_of(decided, n_keep, head, N, d, rank, red) : kKeepGramSlots;
      auto form_gram = [&]() {
        if (slot < kKeepGramSlots) {
          // the chunk sums of k_bf_keep_gram_part, added in chunk order
          const double* gp = gpart + (size_t)slot * kKeepGramChunks * d * d;
          for (int e = threadIdx.x; e < d * d; e += KB_THREADS) {
            double s = 0.0;
            for (int c = 0; c < kKeepGramChunks; ++c) s += gp[(size_t)c * d * d + e];
            W[e] = s;
          }
          __syncthreads();
        } else if (d == 128) {
          gram_rows_f64<T, 8>(Vh, id, n, W);
        } else {
          gram_rows_f64<T, 4>(Vh, id, n, W);
        }
      };
      // G[i][j] -= R[k][i] R[k][j] for i, j > k with row k of the factor in place: 8 x 32 threads, a thread walks rows
      // i = k+1+ty+8a and columns j = k+1+tx+32b (a wave touches two row segments of 256 bytes)
      auto trailing_update = [&](int k) {
        const int ty = threadIdx.x >> 5, tx = threadIdx.x & 31;
        const double* rk = W + k * d;
        for (int i = k + 1 + ty; i < d; i += 8) {
          const double ri = rk[i];
          double* wi = W + i * d;
          for (int j = k + 1 + tx; j < d; j += 32) wi[j] = fma(-ri, rk[j], wi[j]);
        }
      };
      form_gram();
      // sigma_max^2 = lambda_max(G): power iteration on G
      for (int c = threadIdx.x; c < d; c += KB_THREADS) xv[c] = 1.0 / sqrt((double)d) * (1.0 + 0.01 * (c % 7));
      __syncthreads();
      double lam = 0.0;
      for (int it = 0; it < 24; ++it) {
        double part = 0.0;
        if ((int)threadIdx.x < d) {                                // G symmetric: column reads, no bank conflicts
          const double* col = W + threadIdx.x;
          double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
#pragma unroll 4
          for (int c = 0; c < d; c += 4) {
            s0 = fma(col[(c + 0) * d], xv[c + 0], s0); s1 = fma(col[(c + 1) * d], xv[c + 1], s1);
            s2 = fma(col[(c + 2) * d], xv[c + 2], s2); s3 = fma(col[(c + 3) * d], xv[c + 3], s3);
          }
          const double s = (s0 + s1) + (s2 + s3);
          yv[threadIdx.x] = s; part = s * s;
        }
        const double n2 = block_sum(part, red);
        lam = sqrt(n2);
        if (!(lam > 0.0)) break;
        for (int a = threadIdx.x; a < d; a += KB_THREADS) xv[a] = yv[a] / lam;
        __syncthreads();
      }
      const double smax = sqrt(lam);
      const double thr = smax * (double)max(n, d) * kRankEps;     // on singular values
      // Full-rank shortcut (what a head missed by the single-precision certificate usually is): G - thr^2 I is
      // positive definite iff every eigenvalue of G exceeds thr^2, i.e. every singular value of V_keep exceeds thr.
      const bool full = (d == 128) ? shifted_ldl_positive<8>(W, thr * thr, xv, yv) : shifted_ldl_positive<4>(W, thr * thr, xv, yv);
      int r = d;
      if (!full) {
        // diagonally pivoted Cholesky, upper factor kept in the upper triangle (row k, columns >= k)
        for (int c = threadIdx.x; c < d; c += KB_THREADS) perm[c] = c;
        __syncthreads();
        r = 0;
        for (int k = 0; k < d; ++k) {
          if (threadIdx.x < 128) {                                   // largest remaining diagonal entry, lowest index first
            const int i = threadIdx.x;
            const double dv = (i >= k && i < d) ? W[i * d + i] : 0.0;
            uint64_t key = (dv > 0.0) ? ((((uint64_t)__double_as_longlong(dv)) & ~0x7FULL) | (uint64_t)(127 - i)) : 0ULL;
            key = wave_max_u64(key);
            if ((threadIdx.x & 63) == 0) pkey[threadIdx.x >> 6] = key;
          }
          __syncthreads();
          const uint64_t key = pkey[0] > pkey[1] ? pkey[0] : pkey[1];
          const int p = key ? 127 - (int)(key & 0x7F) : k;
          const double piv = W[p * d + p];
          __syncthreads();                                             // pkey is rewritten in the next step
          if (!(piv > 0.0) || !(sqrt(piv) > thr)) break;
          if (p != k) {   // symmetric swap of rows/columns p and k
            for (int c = threadIdx.x; c < d; c += KB_THREADS) { const double t = W[k * d + c]; W[k * d + c] = W[p * d + c]; W[p * d + c] = t; }
            __syncthreads();
            for (int c = threadIdx.x; c < d; c += KB_THREADS) { const double t = W[c * d + k]; W[c * d + k] = W[c * d + p]; W[c * d + p] = t; }
            if (threadIdx.x == 0) { const int t = perm[k]; perm[k] = perm[p]; perm[p] = t; }
            __syncthreads();
          }
          const double rinv = 1.0 / sqrt(piv);
          for (int c = k + threadIdx.x; c < d; c += KB_THREADS) W[k * d + c] *= rinv;                // row k of the factor
          __syncthreads();
          trailing_update(k);
          __syncthreads();
          r = k + 1;
        }
        __syncthreads();
      }
      r_keep = r;
      if (r_keep < d) {
        // rows 0..r-1 of the factor (zero left of the diagonal), columns back in original order
        for (int e = threadIdx.x; e < d * d; e += KB_THREADS) {
          const int i = e / d, c = e - i * d;
          if (i >= r_keep || c < i) W[e] = 0.0;
        }
        __syncthreads();
        // un-permute columns: out[:, perm[c]] = in[:, c]; done row by row through yv
        for (int i = 0; i < r_keep; ++i) {
          for (int c = threadIdx.x; c < d; c += KB_THREADS) yv[perm[c]] = W[i * d + c];
          __syncthreads();
          for (int c = threadIdx.x; c < d; c += KB_THREADS) W[i * d + c] = yv[c];
          __syncthreads();
        }
        r_keep = pivoted_mgs(W, r_keep, d, thr, red, ired);
      }
    }
    active = (r_keep < d) ? 1 : 0;
    if (active) {
      float* bh = basis + (size_t)head * d * d;
      for (int e = threadIdx.x; e < r_keep * d; e += KB_THREADS) bh[e] = (float)W[e];
    }
  }
  (void)lane; (void)wave;
  if (threadIdx.x == 0) {
    HeadState s;
    s.a_keep = a_keep; s.a_del = a_del; s.n_keep = n; s.n_del = n_del; s.r_keep = r_keep; s.active = active;
    s.k_used = 0; s.pad = 0; s.rcr = 0.f; s.ivn = 0.f;
    state[head] = s;
  }
}

// ------------------------------------------------------------------------------------------------
// Head states for the variants of App. D that do not use the retained span (No Projection, Naive Aggregation): the
// demand sums of Eq. 6, r_keep = 0, and every head with retained and deleted rows is active.
__global__ __launch_bounds__(KB_THREADS) void k_bf_plain_state(const float* __restrict__ scores, const int32_t* __restrict__ idx,
                                                               const int32_t* __restrict__ n_keep, int N, int max_budget,
                                                               int rank, HeadState* __restrict__ state, int scs) {
  __shared__ double red[KB_WAVES];
  const int head = blockIdx.x;
  const int n = n_keep[head];
  const float* sc = scores + (size_t)head * scs;
  const int32_t* id = idx + (size_t)head * max_budget;
  double pk = 0.0, pt = 0.0;
  for (int i = threadIdx.x; i < n; i += KB_THREADS) pk += (double)sc[id[i]];
  for (int i = threadIdx.x; i < N; i += KB_THREADS) pt += (double)sc[i];
  const double a_keep = block_sum(pk, red);
  const double a_tot = block_sum(pt, red);
  if (threadIdx.x == 0) {
    HeadState s;
    s.a_keep = a_keep; s.a_del = fmax(a_tot - a_keep, 0.0); s.n_keep = n; s.n_del = N - n; s.r_keep = 0;
    s.active = (rank > 0 && n > 0 && N - n > 0) ? 1 : 0;
    s.k_used = 0; s.pad = 0; s.rcr = 0.f; s.ivn = 0.f;
    state[head] = s;
  }
}

// ------------------------------------------------------------------------------------------------
// del_stats: partial V_del^T V_del, sum_j A_j v_j and ||V_del||^2 over one chunk of tokens
constexpr int DS_THREADS = 256;
constexpr int DS_TOK = 32;

template <typename T>
__global__ __launch_bounds__(DS_THREADS) void k_bf_del_stats(const T* __restrict__ V, const float* __restrict__ scores,
                                                             const int32_t* __restrict__ idx, int N, int d,
                                                             int max_budget, int nstat,
                                                             const HeadState* __restrict__ state,
                                                             const int32_t* __restrict__ n_keep /*non-null: do not read the head states*/,
                                                             float* __restrict__ gram_part, int scs, int kvs) {
  const int head = blockIdx.y, chunk = blockIdx.x;
  const int n = n_keep ? n_keep[head] : state[head].n_keep;
  if (n_keep ? !(n > 0 && n < N) : !state[head].active) return;
  extern __shared__ float Vs[];              // [DS_TOK][d], retained rows zeroed
  __shared__ float wt[DS_TOK];               // score of the token (0 for rows that are not deleted)
  __shared__ int isdel[DS_TOK];              // 1: deleted row of this chunk
  const int32_t* id = idx + (size_t)head * max_budget;
  const T* Vh = V + (size_t)head * kvs * d;
  const float* sc = scores + (size_t)head * scs;
  const int t0 = chunk * kStatChunk, t1 = min(N, t0 + kStatChunk);
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  const int bs = d / 16;
  float acc[8][8];
  for (int a = 0; a < 8; ++a) for (int b = 0; b < 8; ++b) acc[a][b] = 0.f;
  float u = 0.f, su = 0.f, nn = 0.f;         // threads < d: weighted and plain column sums, squared norm share

  for (int tt = t0; tt < t1; tt += DS_TOK) {
    __syncthreads();
    if (threadIdx.x < DS_TOK) {
      const int j = tt + threadIdx.x;
      float wgt = 0.f;
      int del = 0;
      if (j < t1) {
        int lo = 0, hi = n;                  // is j in the ascending retained list?
        while (lo < hi) { const int mid = (lo + hi) >> 1; if (id[mid] < j) lo = mid + 1; else hi = mid; }
        del = !(lo < n && id[lo] == j);
        wgt = del ? sc[j] : 0.f;
      }
      wt[threadIdx.x] = wgt;
      isdel[threadIdx.x] = del;
    }
    __syncthreads();
    for (int e = threadIdx.x; e < DS_TOK * d; e += DS_THREADS) {
      const int i = e / d, c = e - i * d;
      Vs[e] = isdel[i] ? Elem<T>::load(Vh + (size_t)(tt + i) * d + c) : 0.f;
    }
    __syncthreads();
    for (int i = 0; i < DS_TOK; ++i) {
      float av[8], bv[8];
      for (int a = 0; a < bs; ++a) av[a] = Vs[i * d + ty * bs + a];
      for (int b = 0; b < bs; ++b) bv[b] = Vs[i * d + tx * bs + b];
      for (int a = 0; a < bs; ++a) for (int b = 0; b < bs; ++b) acc[a][b] = fmaf(av[a], bv[b], acc[a][b]);
    }
    if ((int)threadIdx.x < d) {
      for (int i = 0; i < DS_TOK; ++i) {
        const float x = Vs[i * d + threadIdx.x];
        const float wgt = wt[i];
        u = fmaf(wgt, x, u);
        su += x;
        nn = fmaf(x, x, nn);
      }
    }
  }
  float* out = gram_part + ((size_t)head * nstat + chunk) * gram_stride(d);
  for (int a = 0; a < bs; ++a) for (int b = 0; b < bs; ++b) out[(ty * bs + a) * d + tx * bs + b] = acc[a][b];
  if ((int)threadIdx.x < d) { out[d * d + threadIdx.x] = u; out[d * d + d + threadIdx.x] = su; }
  // ||V_del||^2 of the chunk: sum over the d column shares, fixed order
  __shared__ float nsh[128];
  __syncthreads();
  if ((int)threadIdx.x < d) nsh[threadIdx.x] = nn;
  __syncthreads();
  if (threadIdx.x == 0) {
    double s = 0.0;
    for (int c = 0; c < d; ++c) s += (double)nsh[c];
    out[d * d + 2 * d] = (float)s;
  }
}

// ------------------------------------------------------------------------------------------------
// finalize: per head, everything after the streaming pass
constexpr int FN_THREADS = 1024;
constexpr int FN_WAVES = FN_THREADS / 64;
constexpr int FN_SWEEPS = kJacobiSweeps;
constexpr int FN_DIRECT_MIN = 20;         // complements at least this wide take the direct leading-eigenpair route when it applies
constexpr int FN_REPLAY_MIN = 64;        // complements at least this wide do not accumulate eigenvectors (see the Jacobi phase)
// Floats of dynamic LDS of the first finalisation launch: room for the d x (d+1) projector and for T and W of every
// complement up to three quarters of d wide (74.5 KB at d = 128, so that two workgroups still share a CU).
__host__ __device__ inline int fn_small_floats(int d) {
  const int mq = 3 * d / 4, a = d * (d + 1), b = 2 * mq * (mq + 1);
  return a > b ? a : b;
}

// Check after a Jacobi sweep, for a workgroup of FN_THREADS threads (all must call): have the rows of the `rank` largest
// diagonal entries of the symmetric mm x mm matrix T (upper triangle current, row stride lt) separated from the rest?
// True when each of those rows has off-diagonal energy of at most tol / 100 and every other row's Gershgorin bound is
// under 0.99 times the smallest of those diagonal entries.  *total receives the off-diagonal energy of the whole of T.
// The arrays are LDS scratch of mm floats.
__device__ __forceinline__ bool jacobi_lead_rows_done(const float* T, int lt, int mm, int rank, float tol, float* dg,
                                                   float* rowe, float* gers, float* lead_min, int* ok, float* total) {
  const int tid = threadIdx.x;
  if (tid < mm) {
    float ro = 0.f, ga = 0.f;
    for (int b = 0; b < mm; ++b) {
      if (b != tid) { const float v = T[min(tid, b) * lt + max(tid, b)]; ro = fmaf(v, v, ro); ga += fabsf(v); }
    }
    const float dgv = T[tid * lt + tid];
    dg[tid] = dgv; rowe[tid] = ro; gers[tid] = dgv + ga;
  }
  if (tid == 0) *ok = 1;
  __syncthreads();
  int rk = mm;
  if (tid < mm) {
    const float mine = dg[tid];
    rk = 0;
    for (int j = 0; j < mm; ++j) { const float o = dg[j]; rk += (o > mine) || (o == mine && j < tid); }
    if (rk < rank && !(rowe[tid] <= 0.01f * tol)) *ok = 0;
    if (rk == rank - 1) *lead_min = mine;
  }
  if (tid == 0) { float t = 0.f; for (int a = 0; a < mm; ++a) t += rowe[a]; *total = t; }
  __syncthreads();
  if (tid < mm && rk >= rank && !(gers[tid] < 0.99f * *lead_min)) *ok = 0;
  __syncthreads();
  return *ok != 0;
}

// Outputs of one head, shared by the two kernels that can finish it: delta, the head state, the diagnostics, and Eq. 7 on
// the retained rows.  uvec (LDS) holds delta when the head is not skipped.  NT threads, all must call.
template <typename T, int NT>
__device__ __forceinline__ void fn_emit(const int head, const int d, const int rank, HeadState st, const int skipped,
                                        const int k_used, const float rcr, const float ivn, const float pcr, const float pc,
                                        const float revr, const float fast_err, const float* uvec,
                                        HeadState* __restrict__ state,
                                        float* __restrict__ delta, float* __restrict__ delta_out, obf_diag_t* __restrict__ diag,
                                        T* __restrict__ V_out, const int max_budget, const float* __restrict__ scores,
                                        const int32_t* __restrict__ idx, const int vflags, const int scs) {
  const int tid = threadIdx.x;
  if (tid < d) {
    const float v = skipped ? 0.f : uvec[tid];
    delta[(size_t)head * d + tid] = v;
    if (delta_out) delta_out[(size_t)head * d + tid] = v;
  }
  if (tid == 0) {
    st.active = skipped ? 0 : 1;
    st.k_used = k_used; st.rcr = rcr; st.ivn = ivn;
    state[head] = st;
    if (diag) {
      obf_diag_t dg;
      dg.n_keep = st.n_keep; dg.r_keep = st.r_keep; dg.k_used = k_used; dg.skipped = skipped;
      dg.a_keep = (float)st.a_keep; dg.a_del = (float)st.a_del; dg.rcr = rcr; dg.ivn = ivn;
      // a head whose retained span is all of R^d has its deleted values entirely inside it
      dg.pcr = (rank > 0 && st.n_keep > 0 && st.n_del > 0 && st.r_keep >= d) ? 1.f : pcr;
      dg.pc = pc; dg.revr = revr;
      dg.dr = (float)(st.a_del / (st.a_keep + kEps));
      dg.fast_err = fast_err;
      dg.select_flags = 0;                                     // the fused call fills it in afterwards
      diag[head] = dg;
    }
  }
  // Eq. 7: the one offset is added to every retained value row (rounded once to the storage type); under Attn-inject
  // (App. D) row t receives n_keep A_t / (a_keep + eps) times the offset instead
  if (!skipped && V_out) {
    const int total = st.n_keep * d;
    T* base = V_out + (size_t)head * max_budget * d;
    if (vflags & VF_ATTN_INJECT) {
      const float per_mass = (float)((double)st.n_keep / (st.a_keep + kEps));
      const float* sc = scores + (size_t)head * scs;
      const int32_t* id = idx + (size_t)head * max_budget;
      for (int e = tid; e < total; e += NT) {
        T* p = base + e;
        Elem<T>::store(p, fmaf(per_mass * sc[id[e / d]], uvec[e % d], Elem<T>::load(p)));
      }
    } else {
      for (int e = tid; e < total; e += NT) {
        T* p = base + e;
        Elem<T>::store(p, Elem<T>::load(p) + uvec[e % d]);
      }
    }
  }
}

template <typename T>
__global__ __launch_bounds__(FN_THREADS, 8) void k_bf_finalize(int N, int d, int nstat, int rank,
                                                            HeadState* __restrict__ state,
                                                            const float* __restrict__ basis,
                                                            const float* __restrict__ gram_part,
                                                            float* __restrict__ mats, float* __restrict__ delta,
                                                            float* __restrict__ delta_out, obf_diag_t* __restrict__ diag,
                                                            T* __restrict__ V_out, int max_budget, int cls,
                                                            const float* __restrict__ scores,
                                                            const int32_t* __restrict__ idx, int vflags, float evr_tau,
                                                            int scs, float* __restrict__ rot /*nullable*/,
                                                            LeadJob* __restrict__ lead /*nullable: no leading-eigenpair kernel follows*/,
                                                            int m_direct_min, int m_direct_max) {
  extern __shared__ float sm[];
  const int head = blockIdx.x;
  const int ld = d + 1;
  float* U = sm;                    // [d][ld]   projector P, then the rows of Z; later T and (if they both fit) W
  float* M = sm;                    // T = Z G Z^T and its diagonal form, set below
  __shared__ __attribute__((aligned(16))) float4 rotp[64];       // (p, q, cos, sin) of each rotation of the current set; p and q as integer bits
  __shared__ float uvec[128], svec[128], rbar[128], dvec[128], lamv[128];
  __shared__ int order[128];
  __shared__ float fred[FN_WAVES];
  __shared__ int s_k;
  __shared__ float s_off;
  __shared__ __attribute__((aligned(16))) float xcol[128], xcol2[128];
  __shared__ uint32_t wkey[2][4];
  HeadState st = state[head];
  int skipped = 1;
  float rcr = 0.f, ivn = 0.f, pcr = 0.f, pc = 0.f, revr = 0.f;
  int k_used = 0;
  const int tid = threadIdx.x;
  const bool naive = (vflags & VF_NAIVE) != 0;
  {
    // Two launches share the heads: the first has fn_small_floats(d) floats of LDS (two workgroups per CU) and takes
    // every head whose complement is small enough for T and W to fit there, the second takes the rest.
    const int m0 = (st.active && !naive) ? d - st.r_keep : 0;
    const int mm0 = m0 + (m0 & 1);
    const int big = 2 * mm0 * (mm0 + 1) > fn_small_floats(d);
    if (cls >= 0 && big != cls) return;                        // cls < 0: one launch with the large LDS takes every head
  }
  if (lead && tid == 0) lead[head].pending = 0;

  if (st.active && naive) {
    // Naive Aggregation (App. D): the plain mean of the deleted value rows, none of Eq. 3-6
    const size_t pstride = gram_stride(d);
    const float* gp = gram_part + (size_t)head * nstat * pstride;
    if (tid < d) {
      float s = 0.f;
      for (int c = 0; c < nstat; ++c) s += gp[c * pstride + d * d + d + tid];
      uvec[tid] = s / (float)st.n_del;
    }
    __syncthreads();
    if (tid == 0) { double s = 0.0; for (int c = 0; c < d; ++c) s += (double)uvec[c] * uvec[c]; s_off = (float)sqrt(s); }
    __syncthreads();
    ivn = s_off;
    skipped = 0;
  }
  if (st.active && !naive) {
    const int r = st.r_keep;
    int m = d - r;                                             // dimension of the orthogonal complement
    const float* Qb = basis + (size_t)head * d * d;            // [r][d] orthonormal rows
    const size_t pstride = gram_stride(d);
    const float* gp = gram_part + (size_t)head * nstat * pstride;
    float* Zg = mats + (size_t)head * 3 * d * d;               // [m][d] basis of the complement (global scratch)
    float* Yg = Zg + (size_t)d * d;                            // [m][d] Z G
    float* Gg = Yg + (size_t)d * d;                            // [d][d] G summed over the chunk partials

    // G = sum of chunk partials (fixed order), u, ||V_del||^2
    // only the 32 x 32 tiles on and below the diagonal of a partial are defined; the sum is mirrored
    for (int e = tid * 4; e < d * d; e += FN_THREADS * 4) {
      const int row = e / d, col = e - row * d;
      if ((row >> 5) < (col >> 5)) continue;
      float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 8
      for (int c = 0; c < nstat; ++c) {
        const float4 q = *(const float4*)(gp + c * pstride + e);
        s.x += q.x; s.y += q.y; s.z += q.z; s.w += q.w;
      }
      *(float4*)(Gg + e) = s;                                  // read back (through L2) when X = G Z^T is formed
      if ((row >> 5) > (col >> 5)) {
        Gg[(col + 0) * d + row] = s.x; Gg[(col + 1) * d + row] = s.y;
        Gg[(col + 2) * d + row] = s.z; Gg[(col + 3) * d + row] = s.w;
      }
    }
    if (tid < d) {
      float s = 0.f;
#pragma unroll 8
      for (int c = 0; c < nstat; ++c) s += gp[c * pstride + d * d + tid];
      uvec[tid] = s;
      float s2 = 0.f;
#pragma unroll 8
      for (int c = 0; c < nstat; ++c) s2 += gp[c * pstride + d * d + d + tid];
      svec[tid] = s2;
    }
    float vd2 = 0.f;
#pragma unroll 8
    for (int c = 0; c < nstat; ++c) vd2 += gp[c * pstride + d * d + 2 * d];

    __syncthreads();                                           // G is in global scratch for every thread of the workgroup
    // P = I - Q^T Q (projector onto the complement of the retained span, Eq. 3) on the matrix cores: wave (rb, cb)
    // holds the 32 x 32 tile of P in 16 registers per lane, entry i of lane l being
    // P[rb*32 + (i/4)*8 + (l/32)*4 + i%4][cb*32 + l%32].
    const int lane = tid & 63, l31 = lane & 31, lh = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int TD = d >> 5;
    // P is symmetric: only the tiles on and below the diagonal are formed and deflated (10 of 16 at d = 128; the waves
    // of the others stay out of the way), and a column's entries above the diagonal block are read off as the row of
    // the mirrored tile
    const bool ptile = wave < TD * TD && wave / TD >= wave % TD;
    const int rb = wave / TD, cb = wave % TD;
    f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    if (ptile) {
      const float* qa = Qb + rb * 32 + l31;
      const float* qb = Qb + cb * 32 + l31;
      for (int k0 = 0; k0 < r; k0 += 16) {                      // eight operand pairs in flight per group
        float av[8], bv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int k = k0 + 2 * u + lh;
          const size_t o = (size_t)min(k, r - 1) * d;
          av[u] = qa[o]; bv[u] = qb[o];
          if (k >= r) { av[u] = 0.f; bv[u] = 0.f; }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u], bv[u], acc, 0, 0, 0);
      }
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int row = rb * 32 + (i >> 2) * 8 + lh * 4 + (i & 3), col = cb * 32 + l31;
        acc[i] = ((row == col) ? 1.f : 0.f) - acc[i];
        if (row == col) xcol[row] = acc[i];
      }
    }
    __syncthreads();

    // Diagonally pivoted Cholesky of P, right-looking on the register tiles: a projector of rank m factors as
    // P = Z^T Z with the m rows of Z orthonormal, i.e. Z is an orthonormal basis of the complement.  A step takes the
    // two columns with the largest remaining diagonals, factors their 2 x 2 block, scales the pair into two rows of Z
    // (LDS) and deflates P by both (one pair of barriers for two rows); when the second column loses most of its
    // diagonal to the first, the step takes the first alone and the choice is made again.
    float dg = (tid < d) ? xcol[tid] : -1.f;
    bool used = false;
    auto publish = [&](int buf) {                              // per wave: its two largest (remaining diagonal, lowest index first)
      if (tid < 128) {
        const uint32_t key = (!used && dg > 0.f) ? ((__float_as_uint(dg) & ~0x7Fu) | (uint32_t)(127 - tid)) : 0u;
        const uint32_t k1 = wave_max_u32(key);
        const uint32_t k2 = wave_max_u32(key == k1 ? 0u : key);  // non-zero keys are distinct: they carry the index
        if (lane == 0) { wkey[buf][2 * (tid >> 6)] = k1; wkey[buf][2 * (tid >> 6) + 1] = k2; }
      }
    };
    __syncthreads();
    publish(0);
    __syncthreads();
    // column j of P to LDS: the tiles of block column j / 32 hold its entries from the diagonal block down in the lanes
    // of that column; the tiles of block row j / 32 left of the diagonal hold the others as row j (one register of the
    // half-wave that owns the row, the same register in every such tile: a jump, not a chain of selects)
    auto put_column = [&](const int j, float* dst) {
      if (!ptile) return;
      const int J = j >> 5, jr = j & 31;
      if (cb == J && l31 == jr) {
#pragma unroll
        for (int i = 0; i < 16; ++i) dst[rb * 32 + (i >> 2) * 8 + lh * 4 + (i & 3)] = acc[i];
      }
      if (rb == J && cb < J && lh == ((jr >> 2) & 1)) {
        float v = 0.f;
        switch ((jr >> 3) * 4 + (jr & 3)) {
#define OBF_FN_CASE(q) case q: v = acc[q]; break;
          OBF_FN_CASE(0) OBF_FN_CASE(1) OBF_FN_CASE(2) OBF_FN_CASE(3) OBF_FN_CASE(4) OBF_FN_CASE(5) OBF_FN_CASE(6) OBF_FN_CASE(7)
          OBF_FN_CASE(8) OBF_FN_CASE(9) OBF_FN_CASE(10) OBF_FN_CASE(11) OBF_FN_CASE(12) OBF_FN_CASE(13) OBF_FN_CASE(14) OBF_FN_CASE(15)
#undef OBF_FN_CASE
          default: break;
        }
        dst[cb * 32 + l31] = v;
      }
    };
    {
      int s = 0, buf = 0;
      while (s < m) {
        const uint32_t a1 = wkey[buf][0], a2 = wkey[buf][1], b1 = wkey[buf][2], b2 = wkey[buf][3];
        const uint32_t key1 = max(a1, b1);
        uint32_t key2 = (a1 > b1) ? max(a2, b1) : max(a1, b2);
        if (key1 == 0u) { m = s; break; }
        if (s + 1 >= m) key2 = 0u;                                // one row left to find
        const int j1 = 127 - (int)(key1 & 0x7Fu), j2 = key2 ? 127 - (int)(key2 & 0x7Fu) : -1;
        put_column(j1, xcol);
        if (j2 >= 0) put_column(j2, xcol2);
        lds_barrier();
        const float p11 = xcol[j1];
        if (!(p11 > 1e-5f)) { m = s; break; }                     // cannot happen for an exact projector of rank m
        const float i1 = rsqrtf(p11);
        float l21 = 0.f, i2 = 0.f;
        bool two = false;
        if (j2 >= 0) {
          const float p22 = xcol2[j2];
          l21 = xcol[j2] * i1;
          const float sc = fmaf(-l21, l21, p22);                  // what the first column leaves of the second diagonal
          two = sc > 1e-5f && sc > 0.25f * p22;
          if (two) i2 = rsqrtf(sc);
        }
        if (ptile) {
          // z1 = x1 i1 and z2 = (x2 - g x1) i2 with g = l21 i1: the deflation z1 z1^T + z2 z2^T of this tile, written
          // on the raw columns so that an entry costs two multiply-adds: x1_r e1_c + x2_r e2_c
          const float x1c = xcol[cb * 32 + l31];
          if (two) {                                              // uniform
            const float g = l21 * i1;
            const float e2 = -(i2 * i2) * fmaf(-g, x1c, xcol2[cb * 32 + l31]);
            const float e1 = fmaf(-(i1 * i1), x1c, -g * e2);
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
              const float4 x1 = *(const float4*)&xcol[rb * 32 + i4 * 8 + lh * 4];
              const float4 x2 = *(const float4*)&xcol2[rb * 32 + i4 * 8 + lh * 4];
              acc[4 * i4 + 0] = fmaf(x1.x, e1, fmaf(x2.x, e2, acc[4 * i4 + 0]));
              acc[4 * i4 + 1] = fmaf(x1.y, e1, fmaf(x2.y, e2, acc[4 * i4 + 1]));
              acc[4 * i4 + 2] = fmaf(x1.z, e1, fmaf(x2.z, e2, acc[4 * i4 + 2]));
              acc[4 * i4 + 3] = fmaf(x1.w, e1, fmaf(x2.w, e2, acc[4 * i4 + 3]));
            }
          } else {
            const float e1 = -(i1 * i1) * x1c;
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
              const float4 x1 = *(const float4*)&xcol[rb * 32 + i4 * 8 + lh * 4];
              acc[4 * i4 + 0] = fmaf(x1.x, e1, acc[4 * i4 + 0]);
              acc[4 * i4 + 1] = fmaf(x1.y, e1, acc[4 * i4 + 1]);
              acc[4 * i4 + 2] = fmaf(x1.z, e1, acc[4 * i4 + 2]);
              acc[4 * i4 + 3] = fmaf(x1.w, e1, acc[4 * i4 + 3]);
            }
          }
        }
        if (tid < d) {
          const float z1 = used ? 0.f : xcol[tid] * i1;           // rows already taken are zero in exact arithmetic
          U[s * ld + tid] = z1;                                   // row s of Z
          float z2 = 0.f;
          if (two) {
            z2 = (used || tid == j1) ? 0.f : (xcol2[tid] - l21 * z1) * i2;
            U[(s + 1) * ld + tid] = z2;
          }
          if (tid == j1 || (two && tid == j2)) used = true;
          if (!used) dg -= fmaf(z1, z1, z2 * z2);
        }
        s += two ? 2 : 1;
        buf ^= 1;
        publish(buf);
        lds_barrier();
      }
    }
    __syncthreads();

    // projection cosine (App. K.2): with s the column sum of V_del, the column sum of V_par is s - Z^T Z s, and
    // their cosine is |s_par| / |s| = sqrt(1 - |Z s|^2 / |s|^2)
    {
      float zs2 = 0.f, sd2 = 0.f;
      if (tid < m) { float z = 0.f; for (int c = 0; c < d; ++c) z = fmaf(U[tid * ld + c], svec[c], z); zs2 = z * z; }
      if (tid < d) sd2 = svec[tid] * svec[tid];
      for (int o = 32; o > 0; o >>= 1) { zs2 += __shfl_xor(zs2, o); sd2 += __shfl_xor(sd2, o); }
      if (tid < 128 && lane == 0) { fred[tid >> 6] = zs2; fred[2 + (tid >> 6)] = sd2; }
      __syncthreads();
      const float z2 = fred[0] + fred[1], s2 = fred[2] + fred[3];
      pc = (s2 > 0.f) ? sqrtf(fmaxf(s2 - z2, 0.f) / s2) : 0.f;
      __syncthreads();
    }
    // Z to global scratch (for the last phase), X = G Z^T (d x m) and T = Z X (m x m) on the matrix cores.
    // T is the residual Gram matrix R^T R = P G P restricted to the complement; its eigenpairs (lambda, w) give
    // those of P G P as (lambda, Z^T w).
    for (int e = tid; e < m * d; e += FN_THREADS) Zg[e] = U[(e / d) * ld + (e % d)];
    const int MB = (m + 31) >> 5, MP = MB << 5;
    float* Xg = Yg;                                              // [d][MP]
    if (wave < TD * MB) {
      const int cblk = wave / MB, tblk = wave % MB;
      const int t = tblk * 32 + l31;
      const float* ga = Gg + cblk * 32 + l31;                    // G symmetric: G[c][b] read as G[b][c], coalesced
      const float* zb = U + min(t, m - 1) * ld;
      f32x16 xa;
#pragma unroll
      for (int i = 0; i < 16; ++i) xa[i] = 0.f;
      for (int k0 = 0; k0 < d; k0 += 16) {
        float av[8], bv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int k = k0 + 2 * u + lh;
          av[u] = ga[(size_t)k * d];
          bv[u] = (t < m) ? zb[k] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) xa = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u], bv[u], xa, 0, 0, 0);
      }
#pragma unroll
      for (int i = 0; i < 16; ++i) Xg[(size_t)(cblk * 32 + (i >> 2) * 8 + lh * 4 + (i & 3)) * MP + t] = xa[i];
    }
    __syncthreads();
    const int mm = m + (m & 1);
    const int lt = mm + 1;
    f32x16 ta;
#pragma unroll
    for (int i = 0; i < 16; ++i) ta[i] = 0.f;
    const int sblk = wave / max(MB, 1), tblk2 = wave % max(MB, 1);
    const bool ttile = wave < MB * MB && sblk >= tblk2;          // T is symmetric: the tiles on and below the diagonal
    if (ttile) {
      const int srow = sblk * 32 + l31;
      const float* za = U + min(srow, m - 1) * ld;
      const float* xb = Xg + tblk2 * 32 + l31;
      for (int k0 = 0; k0 < d; k0 += 16) {
        float av[8], bv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int k = k0 + 2 * u + lh;
          av[u] = (srow < m) ? za[k] : 0.f;
          bv[u] = xb[(size_t)k * MP];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) ta = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u], bv[u], ta, 0, 0, 0);
      }
    }
    __syncthreads();                                             // Z (in LDS) is dead from here on
    U = (2 * mm * lt <= fn_small_floats(d)) ? sm + mm * lt : sm + d * ld;   // W next to T, or in the second buffer of the large launch
    if (ttile) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int srow = sblk * 32 + (i >> 2) * 8 + lh * 4 + (i & 3), t = tblk2 * 32 + l31;
        if (srow < m && t < m) M[srow * lt + t] = ta[i];
      }
    }
    if (mm > m) for (int e = tid; e < mm; e += FN_THREADS) { M[m * lt + e] = 0.f; M[e * lt + m] = 0.f; }
    __syncthreads();
    // symmetrise, W = I, trace
    for (int e = tid; e < mm * mm; e += FN_THREADS) {
      const int a = e / mm, b = e - a * mm;
      if (a < b) M[a * lt + b] = M[b * lt + a];                  // the upper triangle mirrors the computed lower one
      U[a * lt + b] = (a == b) ? 1.f : 0.f;
    }
    __syncthreads();
    if (wave == 0) {                                             // trace(T) = ||R||_F^2, summed in double
      double tr = (lane < m) ? (double)M[lane * lt + lane] : 0.0;
      if (lane + 64 < m) tr += (double)M[(lane + 64) * lt + lane + 64];
      for (int o = 32; o > 0; o >>= 1) tr += __shfl_xor(tr, o);
      if (lane == 0) s_off = (float)tr;
    }
    __syncthreads();
    const float res2 = s_off;
    rcr = res2 / (vd2 + 1e-12f);
    pcr = fmaxf(vd2 - res2, 0.f) / (vd2 + 1e-12f);
    const bool negligible = !(res2 > kRcrSkip * vd2) || m <= 0;

    // Only a few leading eigenpairs wanted (the method itself: k = pca_rank, no Max-P / EVR rule) from a wide enough
    // complement: the head is handed to the leading-eigenpair kernel (tridiagonalisation + bisection + inverse iteration,
    // with a register budget of its own) instead of diagonalising all of T here.
    const int kq = min(rank, m);
    const bool direct = lead != nullptr && !negligible && !(vflags & (VF_SUBSPACE_ALL | VF_SUBSPACE_EVR)) && kq >= 1 &&
                        kq <= TE_MAXK && m >= m_direct_min && m <= m_direct_max;
    if (direct) {
      float* Tg = Gg;                                            // G itself is no longer needed
      for (int e = tid; e < m * m; e += FN_THREADS) { const int a = e / m; Tg[e] = M[a * lt + (e - a * m)]; }
      if (tid < d) delta[(size_t)head * d + tid] = uvec[tid];    // u = sum_j A_j v_j; the other kernel replaces it by delta
      if (tid == 0) {
        LeadJob jb;
        jb.pending = 1; jb.m = m; jb.res2 = res2; jb.vd2 = vd2; jb.pc = pc; jb.pcr = pcr; jb.rcr = rcr; jb.pad = 0;
        lead[head] = jb;
      }
      return;
    }
    if (!negligible && !direct) {
      // cyclic Jacobi with a round-robin ordering: mm/2 disjoint rotations per round
      const int half = mm / 2;
      // Wide complements: only W_k W_k^T y is needed of the eigenvectors (y = Z u, W_k the k_used leading ones), and
      // W is the product of all rotations.  Instead of carrying the m x m matrix W through every rotation set (most
      // of a set's work when m is large), the tangents are stored, y is rotated along (z = W^T y costs two entries
      // per rotation), and afterwards the kept coordinates of z are taken back through the rotations in reverse order
      // by one wave.  The result is the same product of the same rotations.
      const bool replay = rot != nullptr && mm >= FN_REPLAY_MIN;
      float* rot_h = rot ? rot + (size_t)head * FN_SWEEPS * (d - 1) * (d / 2) : nullptr;
      int nsweeps = 0;
      // z = W^T y travels with the rotations in the registers of the lanes that compute them: in set r lane i >= 1
      // holds z[(r + i) mod (mm-1)] and z[(r - i) mod (mm-1)], lane 0 holds z[mm-1] and z[r]
      float za = 0.f, zb = 0.f;
      if (replay) {
        if (tid < mm) {
          float s = 0.f;
          if (tid < m) for (int c = 0; c < d; ++c) s = fmaf(Zg[(size_t)tid * d + c], uvec[c], s);
          rbar[tid] = s;                                       // y = Z u
        }
        __syncthreads();
        if (tid < half) { za = rbar[tid == 0 ? mm - 1 : tid]; zb = rbar[tid == 0 ? 0 : mm - 1 - tid]; }
      }
      auto rot_of = [&](const float* A, const int p, const int q, float& c, float& s, float& tt) {
        const float app = A[__mul24(p, lt) + p], aqq = A[__mul24(q, lt) + q], apq = A[__mul24(p, lt) + q];
        c = 1.f; s = 0.f; tt = 0.f;
        // single-instruction reciprocal / square roots (1 ulp): the rotation only has to be orthogonal to rounding
        if (fabsf(apq) > 1e-30f && fabsf(apq) > 1e-9f * __builtin_amdgcn_sqrtf(fabsf(app * aqq)) ) {
          const float tau = (aqq - app) * __builtin_amdgcn_rcpf(2.f * apq);
          const float t = copysignf(__builtin_amdgcn_rcpf(fabsf(tau) + __builtin_amdgcn_sqrtf(fmaf(tau, tau, 1.f))), tau);
          c = __builtin_amdgcn_rsqf(fmaf(t, t, 1.f));
          s = t * c;
          tt = t;
        }
      };
      // The work items of a rotation set: the 2 x 2 blocks (i, j), i <= j, of T - at most three per thread, found once
      // (item e of the triangle walked by rows) - and the half x mm (rotation, row) pairs of W, walked with a stride of
      // FN_THREADS by fixed index steps.  The sets contain no division.
      const int nw = half * mm;
      int items[3];
#pragma unroll
      for (int u = 0; u < 3; ++u) {
        const int e = tid + u * FN_THREADS;
        items[u] = -1;
        if (e < half * (half + 1) / 2) {
          int i = 0, rem = e;
          while (rem >= half - i) { rem -= half - i; ++i; }
          items[u] = i | ((i + rem) << 16);
        }
      }
      const int wi0 = tid / max(mm, 1), wk0 = tid - wi0 * mm, wdi = FN_THREADS / max(mm, 1), wdk = FN_THREADS - wdi * mm;
      // One 2 x 2 block of a rotation set.  Only the upper triangle of T is kept current during the sweeps: entry
      // (x, y) lives at (min, max).
      struct RotBlock { int e_a, e_b, e_c, e_d; float a, b, c, dd, ci, si, cj, sj; bool diag; };
      auto block_load = [&](const int item, RotBlock& k) {
        const int i = item & 0xffff, jb = item >> 16;
        const float4 ri = rotp[i], rj = rotp[jb];
        const int p = __float_as_int(ri.x), q = __float_as_int(ri.y), p2 = __float_as_int(rj.x), q2 = __float_as_int(rj.y);
        k.ci = ri.z; k.si = ri.w; k.cj = rj.z; k.sj = rj.w;
        k.diag = i == jb;
        // 24-bit multiplies (full rate; the indices are below 2^7)
        k.e_a = __mul24(min(p, p2), lt) + max(p, p2); k.e_b = __mul24(min(p, q2), lt) + max(p, q2);
        k.e_c = k.diag ? k.e_b : __mul24(min(q, p2), lt) + max(q, p2); k.e_d = __mul24(min(q, q2), lt) + max(q, q2);
        k.a = M[k.e_a]; k.b = M[k.e_b]; k.c = M[k.e_c]; k.dd = M[k.e_d];
      };
      auto block_store = [&](const RotBlock& k) {
        const float a1 = k.cj * k.a - k.sj * k.b, b1 = k.sj * k.a + k.cj * k.b, c1 = k.cj * k.c - k.sj * k.dd, d1 = k.sj * k.c + k.cj * k.dd;
        const float a2 = k.ci * a1 - k.si * c1, c2 = k.si * a1 + k.ci * c1, b2 = k.ci * b1 - k.si * d1, d2 = k.si * b1 + k.ci * d1;
        if (k.diag) {
          M[k.e_a] = a2; M[k.e_d] = d2; M[k.e_b] = 0.5f * (b2 + c2);
        } else {
          M[k.e_a] = a2; M[k.e_b] = b2; M[k.e_c] = c2; M[k.e_d] = d2;
        }
      };
      const bool two_items = __builtin_amdgcn_ballot_w64(items[1] >= 0) != 0;      // wave-uniform
      for (int sweep = 0; sweep < FN_SWEEPS && mm > 1; ++sweep) {
        for (int round = 0; round < mm - 1; ++round) {
          if (tid < half) {
            int p, q;
            if (tid == 0) { p = mm - 1; q = round; }
            else {                                                // (round + tid) mod (mm-1), (round - tid) mod (mm-1); tid < mm-1
              p = round + tid; if (p >= mm - 1) p -= mm - 1;
              q = round - tid; if (q < 0) q += mm - 1;
            }
            const bool swapped = p > q;
            if (swapped) { const int t = p; p = q; q = t; }
            float c, s, t;
            rot_of(M, p, q, c, s, t);
            rotp[tid] = make_float4(__int_as_float(p), __int_as_float(q), c, s);
            if (replay) {
              rot_h[((size_t)sweep * (mm - 1) + round) * half + tid] = t;
              // z <- J^T z on the pair this lane holds (the rotation is defined on the sorted pair), then the step to
              // the next set: first entries one lane down, second entries one lane up, lane 1's first entry into
              // lane 0's second, the last lane's second entry into its first
              const float se = swapped ? -s : s;
              const float na = fmaf(-se, zb, c * za), nb = fmaf(se, za, c * zb);
              const float da = wave_from_above(na), ub = wave_from_below(nb);
              za = (tid == 0) ? na : (tid == half - 1) ? nb : da;
              zb = (tid == 0) ? da : ub;
            }
          }
          // the two barriers of a set wait for LDS traffic only: the tangent stores (read back by the same wave after
          // the sweeps, behind full barriers) stay in flight
          lds_barrier();
          // T <- J^T T J by 2 x 2 blocks (rows {p_i, q_i} x columns {p_j, q_j}, i <= j: the blocks are disjoint, so one
          // pass does both sides), and W <- W J by columns
          if (two_items) {
            // waves in which some thread has a second block: both blocks' loads are issued before the first one's
            // arithmetic (a thread without a second block repeats the loads of its first and drops the result)
            RotBlock k0, k1;
            const bool v1 = items[1] >= 0;
            block_load(items[0], k0);
            block_load(v1 ? items[1] : items[0], k1);
            block_store(k0);
            if (v1) block_store(k1);
          } else if (items[0] >= 0) {
            RotBlock k0;
            block_load(items[0], k0);
            block_store(k0);
          }
          if (items[2] >= 0) {
            RotBlock k2;
            block_load(items[2], k2);
            block_store(k2);
          }
          for (int e = tid, i = wi0, k = wk0; e < nw && !replay; e += FN_THREADS) {
            const float4 ri = rotp[i];
            const int p = __float_as_int(ri.x), q = __float_as_int(ri.y);
            const float c = ri.z, s = ri.w;
            const int kr = __mul24(k, lt);
            const float wp = U[kr + p], wq = U[kr + q];
            U[kr + p] = c * wp - s * wq;
            U[kr + q] = s * wp + c * wq;
            i += wdi; k += wdk;
            if (k >= mm) { k -= mm; ++i; }
          }
          lds_barrier();
        }
        // The sweeps stop when the off-diagonal energy is below single-precision noise of the trace.  Where only a few
        // leading eigenpairs are used (no Max-P / EVR rule, rank <= mm/8) they also stop as soon as the rows of the
        // `rank` largest diagonal entries are each a hundred times further below that level and every other row's
        // Gershgorin bound stays under the smallest of them by 1 %: those diagonal entries are then the leading
        // eigenvalues and their rotations' columns the eigenvectors, to the same residual as at full convergence,
        // whatever the rest of T still looks like.
        const float tol = 1e-13f * res2 * res2;
        const bool lead_only = !(vflags & (VF_SUBSPACE_ALL | VF_SUBSPACE_EVR)) && 8 * rank <= mm;
        bool lead_done = false;
        if (lead_only) {
          lead_done = jacobi_lead_rows_done(M, lt, mm, rank, tol, lamv, svec, dvec, &fred[1], &s_k, &s_off);
        } else {
          float off = 0.f;
          for (int e = tid; e < mm * mm; e += FN_THREADS) {
            const int a = e / mm, b = e - a * mm;
            if (a < b) { const float v = M[a * lt + b]; off = fmaf(2.f * v, v, off); }
          }
          for (int o = 32; o > 0; o >>= 1) off += __shfl_xor(off, o);
          if ((tid & 63) == 0) fred[tid >> 6] = off;
          __syncthreads();
          if (tid == 0) { float t = 0.f; for (int i = 0; i < FN_WAVES; ++i) t += fred[i]; s_off = t; }
          __syncthreads();
        }
        const float offn = s_off;
        __syncthreads();
        nsweeps = sweep + 1;
        if (offn <= tol || lead_done) break;
      }
      if (replay && tid < half) {                              // whole sweeps end in the layout of set 0
        rbar[tid == 0 ? mm - 1 : tid] = za;
        rbar[tid == 0 ? 0 : mm - 1 - tid] = zb;
      }
      // eigenvalues, descending order (ties: lower index first), numerical rank of R
      if (tid < m) lamv[tid] = M[tid * lt + tid];
      __syncthreads();
      if (tid < m) {
        const float mine = lamv[tid];
        int rk = 0;
        for (int j = 0; j < m; ++j) { const float o = lamv[j]; rk += (o > mine) || (o == mine && j < tid); }
        order[rk] = tid;
      }
      __syncthreads();
      if (tid == 0) {
        const float lmax = lamv[order[0]];
        const float srel = (float)max(st.n_del, d) * (float)kRankEps;
        const float floor_rel = fmaxf(srel * srel, kEigFloor);
        int rankR = 0;
        for (int j = 0; j < m; ++j) if (lamv[order[j]] > lmax * floor_rel) ++rankR;
        const int cap = min(min(st.n_del, d - r), d);
        if (rankR > cap) rankR = cap;
        int want = rank;
        if (vflags & VF_SUBSPACE_ALL) want = d;                  // Max-P (App. D): every direction of R
        if (vflags & VF_SUBSPACE_EVR) {                          // EVR-adaptive rank (App. D)
          double tot = 0.0, cum = 0.0;
          for (int j = 0; j < m; ++j) tot += (double)fmaxf(lamv[order[j]], 0.f);
          want = m;
          for (int j = 0; j < m; ++j) {
            cum += (double)fmaxf(lamv[order[j]], 0.f);
            if (cum >= (double)evr_tau * tot) { want = j + 1; break; }
          }
        }
        s_k = min(want, rankR);
        double top = 0.0;                                        // explained variance of the directions used (App. K.2)
        for (int j = 0; j < s_k; ++j) top += (double)lamv[order[j]];
        s_off = (float)(top / ((double)res2 + 1e-12));
      }
      __syncthreads();
      k_used = s_k;
      revr = (k_used > 0) ? s_off : 0.f;
      __syncthreads();
      if (k_used > 0) {
       if (replay) {
        // x = W D z with D keeping the k_used leading coordinates: the rotations in reverse order, x <- J x, by wave 0.
        // x stays in registers: in set r lane i >= 1 holds x[(r + i) mod nr] and x[(r - i) mod nr] - the pair of its
        // rotation - and lane 0 holds x[nr] and x[r]; stepping to set r - 1 moves the first entries one lane up and the
        // second ones one lane down, with lane 0's second entry entering the first row at lane 1 and the first entry
        // of the last lane entering the second row.
        if (tid < mm) dvec[tid] = 0.f;
        __syncthreads();
        if (tid < k_used) dvec[order[tid]] = rbar[order[tid]];
        __syncthreads();
        // The tangents come back from global memory one sweep at a time through two LDS buffers (T's storage is free
        // by now: its diagonal sits in lamv): while wave 0 replays a sweep, the other waves fetch the one before it.
        {
          const int nr = mm - 1, per = nr * half;
          float* tbuf = sm;
          for (int e = tid; e < per; e += FN_THREADS) tbuf[((nsweeps - 1) & 1) * per + e] = rot_h[(size_t)(nsweeps - 1) * per + e];
          int ia = (tid == 0) ? nr : (nr - 1 + tid) % nr, ib = (tid == 0) ? nr - 1 : (2 * nr - 1 - tid) % nr;   // at r = nr - 1
          float xa = (tid < half) ? dvec[ia] : 0.f, xb = (tid < half) ? dvec[ib] : 0.f;
          __syncthreads();
          for (int sw = nsweeps - 1; sw >= 0; --sw) {
            if (tid >= 64) {
              if (sw > 0) {
                float* dst = tbuf + ((sw - 1) & 1) * per;
                const float* src = rot_h + (size_t)(sw - 1) * per;
                for (int e = tid - 64; e < per; e += FN_THREADS - 64) dst[e] = src[e];
              }
            } else {
              const float* tcur = tbuf + (sw & 1) * per;
              for (int r0 = nr - 1; r0 >= 0; r0 -= 16) {
                float tb[16];                                  // the tangents of sixteen sets are fetched together
#pragma unroll
                for (int u = 0; u < 16; ++u) tb[u] = (r0 - u >= 0 && tid < half) ? tcur[(r0 - u) * half + tid] : 0.f;
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                  if (r0 - u >= 0) {
                    const float t = tb[u];
                    const float c = __builtin_amdgcn_rsqf(fmaf(t, t, 1.f)), s0 = t * c;
                    const float s = (ia < ib) ? s0 : -s0;        // the rotation is defined on the sorted pair
                    const float na = fmaf(s, xb, c * xa), nb = fmaf(-s, xa, c * xb);
                    const float ua = wave_from_below(na), ub = wave_from_below(nb), db = wave_from_above(nb);
                    xa = (tid == 0) ? na : (tid == 1) ? ub : ua;
                    xb = (tid == half - 1) ? na : db;
                    if (tid != 0) ia = (ia == 0) ? nr - 1 : ia - 1;
                    ib = (ib == 0) ? nr - 1 : ib - 1;
                  }
                }
              }
            }
            __syncthreads();
          }
          if (tid < half) { dvec[ia] = xa; dvec[ib] = xb; }
        }
        __syncthreads();
        if (tid < m) lamv[tid] = dvec[tid];                    // Delta in complement coordinates (times a_del + eps)
        __syncthreads();
       } else {
        // In complement coordinates: y = Z u, so that rbar = Z^T y / (a_del + eps)  (Eq. 4 with R_j = P v_j)
        if (tid < m) {
          float s = 0.f;
          for (int c = 0; c < d; ++c) s = fmaf(Zg[(size_t)tid * d + c], uvec[c], s);
          rbar[tid] = s;
        }
        __syncthreads();
        // Delta = sum_i (rbar . c_i) c_i  (Eq. 5) with c_i = Z^T w_i, w_i = column order[i] of W
        if (tid < k_used) {
          const int col = order[tid];
          float s = 0.f;
          for (int t = 0; t < m; ++t) s = fmaf(rbar[t], U[t * lt + col], s);
          dvec[tid] = s;                                   // coefficient
        }
        __syncthreads();
        if (tid < m) {
          float s = 0.f;
          for (int i = 0; i < k_used; ++i) s = fmaf(dvec[i], U[tid * lt + order[i]], s);
          lamv[tid] = s;                                   // Delta in complement coordinates (times a_del + eps)
        }
        __syncthreads();
       }
      }
    }
    if (!negligible && k_used > 0) {
      if (tid < d) {
        float s = 0.f;
        for (int t = 0; t < m; ++t) s = fmaf(Zg[(size_t)t * d + tid], lamv[t], s);
        const double alpha = (vflags & VF_NO_SCALING) ? 1.0 : st.a_del / (st.a_keep + kEps);          // Eq. 6
        uvec[tid] = (float)(alpha * ((double)s / (st.a_del + kEps)));
      }
      __syncthreads();
      if (tid == 0) { double s = 0.0; for (int c = 0; c < d; ++c) s += (double)uvec[c] * uvec[c]; s_off = (float)sqrt(s); }
      __syncthreads();
      ivn = s_off;
      skipped = 0;
    }
  }
  fn_emit<T, FN_THREADS>(head, d, rank, st, skipped, k_used, rcr, ivn, pcr, pc, revr, -1.f, uvec, state, delta, delta_out, diag, V_out,
                         max_budget, scores, idx, vflags, scs);
}

// ------------------------------------------------------------------------------------------------
// The heads the finalisation handed over: leading eigenpairs of T by the direct route, then Eq. 4-7 as there.
// iters > 0 selects the fast path of App. H instead: `iters` steps of C <- orth(C G) from a fixed orthonormal start,
// carried out in complement coordinates (G = Z^T T Z, so a row c of C is followed as its coordinates c Z^T and
// C G becomes Y T); the direct route then runs only when diagnostics are wanted, to report how far the fast path's
// Delta is from it.
template <typename T>
__global__ __launch_bounds__(TE_THREADS, 4) void k_bf_lead(int d, int rank, HeadState* __restrict__ state, float* __restrict__ mats,
                                                          float* __restrict__ delta, float* __restrict__ delta_out,
                                                          obf_diag_t* __restrict__ diag, T* __restrict__ V_out, int max_budget,
                                                          const float* __restrict__ scores, const int32_t* __restrict__ idx,
                                                          int vflags, int scs, const LeadJob* __restrict__ lead, int iters) {
  extern __shared__ float sm[];
  __shared__ float uvec[128], rbar[128], dvec[16], dcomp[128], dex[128];
  __shared__ int s_k;
  __shared__ float s_off;
  const int head = blockIdx.x;
  const LeadJob jb = lead[head];
  if (!jb.pending) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const HeadState st = state[head];
  const int m = jb.m, r = st.r_keep;
  const int lt = m | 1;                                        // odd row stride: column accesses without bank conflicts
  const float* Zg = mats + (size_t)head * 3 * d * d;           // [m][d] basis of the complement
  const float* Tg = Zg + 2 * (size_t)d * d;                    // [m][m]
  float* Rf = sm;
  float* work = sm + ((m * lt + 3) & ~3);                      // 16-byte aligned
  const int kq = min(rank, m);
  if (tid < d) uvec[tid] = delta[(size_t)head * d + tid];      // u
  __syncthreads();
  for (int t0 = wave; t0 < m; t0 += 4 * TE_WAVES) {            // y = Z u (Eq. 4 in complement coordinates), a wave per row,
    float z0[4], z1[4];                                        // four rows' loads in flight
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int t = min(t0 + q * TE_WAVES, m - 1);
      z0[q] = (lane < d) ? Zg[(size_t)t * d + lane] : 0.f;
      z1[q] = (lane + 64 < d) ? Zg[(size_t)t * d + lane + 64] : 0.f;
    }
    const float u0 = (lane < d) ? uvec[lane] : 0.f, u1 = (lane + 64 < d) ? uvec[lane + 64] : 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float sy = te_wave_sum(fmaf(z1[q], u1, z0[q] * u0));
      if (lane == 0 && t0 + q * TE_WAVES < m) rbar[t0 + q * TE_WAVES] = sy;
    }
  }
  // Delta in complement coordinates (times a_del + eps) from kk orthonormal rows Cb [kk][m]: Eq. 5
  auto project = [&](const float* Cb, const int kk) {
    for (int v = wave; v < kk; v += TE_WAVES) {
      float sc = (lane < m) ? rbar[lane] * Cb[v * m + lane] : 0.f;
      if (lane + 64 < m) sc = fmaf(rbar[lane + 64], Cb[v * m + lane + 64], sc);
      sc = te_wave_sum(sc);
      if (lane == 0) dvec[v] = sc;
    }
    __syncthreads();
    if (tid < m) {
      float sd = 0.f;
      for (int i = 0; i < kk; ++i) sd = fmaf(dvec[i], Cb[i * m + tid], sd);
      dcomp[tid] = sd;
    }
    __syncthreads();
  };
  // Per-token alternative (App. D): the subspace goes to the head's second scratch matrix in head_dim coordinates
  // (row i: sum_t Cb[i][t] Z[t][:]) for the kernel that forms the per-slot directions.
  auto export_basis = [&](const float* Cb, const int kk) {
    if (!(vflags & VF_PER_TOKEN)) return;
    float* Cg = mats + ((size_t)head * 3 + 1) * d * d;
    for (int e = tid; e < kk * d; e += TE_THREADS) {
      const int i = e / d, c = e - i * d;
      float s = 0.f;
      for (int t = 0; t < m; ++t) s = fmaf(Cb[i * m + t], Zg[(size_t)t * d + c], s);
      Cg[e] = s;
    }
  };
  int k_used = 0;
  float revr = 0.f, fast_err = -1.f;
  if (iters <= 0 || diag != nullptr) {
    const float* th;
    const float* Wk;
    if (kq <= 4) tri_top_eigs<4>(Tg, m, Rf, lt, m, kq, work, &th, &Wk);
    else tri_top_eigs<8>(Tg, m, Rf, lt, m, kq, work, &th, &Wk);
    if (tid == 0) {
      const float lmax = th[0];
      const float srel = (float)max(st.n_del, d) * (float)kRankEps;
      const float floor_rel = fmaxf(srel * srel, kEigFloor);
      int rankR = 0;
      for (int j = 0; j < kq; ++j) if (th[j] > lmax * floor_rel) ++rankR;      // descending: the count is a prefix
      rankR = min(rankR, min(min(st.n_del, d - r), d));
      s_k = min(rank, rankR);
      double top = 0.0;
      for (int j = 0; j < s_k; ++j) top += (double)th[j];
      s_off = (float)(top / ((double)jb.res2 + 1e-12));
    }
    __syncthreads();
    k_used = s_k;
    revr = (k_used > 0) ? s_off : 0.f;
    __syncthreads();
    project(Wk, k_used);
    if (iters <= 0) export_basis(Wk, k_used);
  }
  if (iters > 0) {
    if (diag != nullptr && tid < m) dex[tid] = dcomp[tid];     // the direct route's Delta, for the error report
    __syncthreads();                                           // the direct route's LDS is free
    float* Tl = sm;                                            // [m][lt]
    float* Ya = work;                                          // [TE_MAXK][m] the current rows
    float* Yb = Ya + TE_MAXK * m;                              // [TE_MAXK][m] their images under T
    float* c0 = work + tri_work_floats(m, kq);                 // [k][d] start rows (the host sized the LDS for them)
    const int k0 = min(min(rank, m), st.n_del);
    for (int e = tid; e < m * m; e += TE_THREADS) { const int a = e / m; Tl[a * lt + (e - a * m)] = Tg[e]; }
    // C_0: the first rows of the orthonormal cosine basis, C_0[i][c] = sqrt(2/d) cos(pi (i + 1/2)(c + 1/2) / d)
    for (int e = tid; e < k0 * d; e += TE_THREADS) {
      const int i = e / d, c = e - i * d;
      c0[e] = sqrtf(2.f / (float)d) * cospif((float)((2 * i + 1) * (2 * c + 1)) / (float)(4 * d));
    }
    __syncthreads();
    for (int v = wave; v < k0; v += TE_WAVES) {
      for (int t = lane; t < m; t += 64) {
        float sy = 0.f;
        for (int c = 0; c < d; ++c) sy = fmaf(c0[v * d + c], Zg[(size_t)t * d + c], sy);
        Ya[v * m + t] = sy;
      }
    }
    if (tid == 0) s_k = k0;
    __syncthreads();
    auto times_T = [&](const int kk) {                         // Yb = Ya T (T is symmetric: row s is read as column s)
      for (int v = wave; v < kk; v += TE_WAVES) {
        float a0 = 0.f, a1 = 0.f;
        for (int s = 0; s < m; ++s) {
          const float ys = Ya[v * m + s];
          a0 = fmaf(ys, (lane < m) ? Tl[s * lt + lane] : 0.f, a0);
          a1 = fmaf(ys, (lane + 64 < m) ? Tl[s * lt + lane + 64] : 0.f, a1);
        }
        if (lane < m) Yb[v * m + lane] = a0;
        if (lane + 64 < m) Yb[v * m + lane + 64] = a1;
      }
      __syncthreads();
    };
    for (int it = 0; it < iters; ++it) {
      const int kk = s_k;
      __syncthreads();
      if (kk == 0) break;                                      // uniform
      times_T(kk);
      if (wave == 0) {
        // orth: Gram-Schmidt over the rows in order, two passes each; a row left with at most 1e-5 of the first row's
        // norm depends on the rows before it and is dropped
        int nk = 0;
        float first = -1.f;
        for (int i = 0; i < kk; ++i) {
          float x0 = (lane < m) ? Yb[i * m + lane] : 0.f, x1 = (lane + 64 < m) ? Yb[i * m + lane + 64] : 0.f;
          for (int pass = 0; pass < 2; ++pass) {
            for (int j = 0; j < nk; ++j) {
              const float y0 = (lane < m) ? Ya[j * m + lane] : 0.f, y1 = (lane + 64 < m) ? Ya[j * m + lane + 64] : 0.f;
              const float dt = te_wave_sum(fmaf(x0, y0, x1 * y1));
              x0 = fmaf(-dt, y0, x0); x1 = fmaf(-dt, y1, x1);
            }
          }
          const float nn = sqrtf(te_wave_sum(fmaf(x0, x0, x1 * x1)));
          if (first < 0.f) first = nn;
          if (!(first > 0.f) || !(nn > 1e-5f * first)) continue;
          const float rn = 1.f / nn;
          if (lane < m) Ya[nk * m + lane] = x0 * rn;
          if (lane + 64 < m) Ya[nk * m + lane + 64] = x1 * rn;
          ++nk;
        }
        if (lane == 0) s_k = nk;
      }
      __syncthreads();
    }
    k_used = s_k;
    __syncthreads();
    revr = 0.f;
    if (k_used > 0) {
      times_T(k_used);                                         // explained share: sum_i c_i T c_i^T over the trace
      for (int v = wave; v < k_used; v += TE_WAVES) {
        float sc = (lane < m) ? Ya[v * m + lane] * Yb[v * m + lane] : 0.f;
        if (lane + 64 < m) sc = fmaf(Ya[v * m + lane + 64], Yb[v * m + lane + 64], sc);
        sc = te_wave_sum(sc);
        if (lane == 0) dvec[v] = sc;
      }
      __syncthreads();
      if (tid == 0) {
        double top = 0.0;
        for (int i = 0; i < k_used; ++i) top += (double)dvec[i];
        s_off = (float)(top / ((double)jb.res2 + 1e-12));
      }
      __syncthreads();
      revr = s_off;
      __syncthreads();
      project(Ya, k_used);
      export_basis(Ya, k_used);
    } else {
      if (tid < m) dcomp[tid] = 0.f;
      __syncthreads();
    }
    if (diag != nullptr) {
      if (tid == 0) {
        double num = 0.0, den = 0.0;
        for (int t = 0; t < m; ++t) { const double e = (double)dcomp[t] - dex[t]; num += e * e; den += (double)dex[t] * dex[t]; }
        s_off = (den > 0.0) ? (float)sqrt(num / den) : 0.f;
      }
      __syncthreads();
      fast_err = s_off;
      __syncthreads();
    }
  }
  int skipped = 1;
  float ivn = 0.f;
  if (k_used > 0) {
    float dl = 0.f;
    if (tid < d) {
      float s = 0.f;
      for (int t = 0; t < m; ++t) s = fmaf(Zg[(size_t)t * d + tid], dcomp[t], s);
      const double alpha = (vflags & VF_NO_SCALING) ? 1.0 : st.a_del / (st.a_keep + kEps);          // Eq. 6
      dl = (float)(alpha * ((double)s / (st.a_del + kEps)));
    }
    __syncthreads();                                           // every thread has read u
    if (tid < d) uvec[tid] = dl;
    __syncthreads();
    if (tid == 0) { double s = 0.0; for (int c = 0; c < d; ++c) s += (double)uvec[c] * uvec[c]; s_off = (float)sqrt(s); }
    __syncthreads();
    ivn = s_off;
    skipped = 0;
  }
  fn_emit<T, TE_THREADS>(head, d, rank, st, skipped, k_used, jb.rcr, ivn, jb.pcr, jb.pc, revr, fast_err, uvec, state, delta, delta_out,
                         diag, V_out, max_budget, scores, idx, vflags, scs);
}

// ------------------------------------------------------------------------------------------------
// host side
// True when the basis of the retained span may be computed beside the gather and the statistics pass: with every
// budget below the head dimension each head with deleted rows is active whatever its basis turns out to be.
static bool basis_overlaps(const Dims& m, int32_t max_budget, int32_t rank) { return rank > 0 && max_budget < m.d; }

// Forks `aux` off `st` and computes the bases there.  *started tells the caller to pass basis_started
// to launch_backfill, which joins `aux` back before the finalisation.
obf_status_t launch_backfill_basis(const Dims& m, const Workspace& w, char* ws, const void* V, const float* scores,
                                   const int32_t* idx, const int32_t* n_keep, int32_t max_budget, int32_t rank,
                                   hipStream_t st, hipStream_t aux, bool* started) {
  *started = false;
  if (!aux || aux == st || !basis_overlaps(m, max_budget, rank)) return OBF_OK;   // no second stream: `st` does it all
  HeadState* state = (HeadState*)(ws + w.head_state);
  float* basis = (float*)(ws + w.basis);
  if (stream_after(aux, st, EV_BASIS_FORK) != OBF_OK) return OBF_ERR_HIP;
  *started = true;                                               // from here on `aux` must be joined, whatever happens
  ProfScope prof_(ST_KEEP_BASIS, aux);
  return launch_keep_basis_small(m, V, scores, idx, n_keep, max_budget, rank, state, basis, aux);
}

template <typename T>
static obf_status_t run(const Dims& m, const Workspace& w, char* ws, const void* V, const float* scores,
                        const int32_t* idx, const int32_t* n_keep, int32_t max_budget, int32_t rank, void* V_out,
                        float* delta_out, obf_diag_t* diag, hipStream_t st, hipStream_t aux, const double* fro_part,
                        bool basis_started, int32_t min_budget, Variant var) {
  // Once the bases run on `aux`, every way out of this function joins it back into `st` first, errors included: the
  // caller is promised that all work of the call is ordered on its stream.
  struct Join {
    hipStream_t st, aux; bool armed;
    obf_status_t now() { if (!armed) return OBF_OK; armed = false; return stream_after(st, aux, EV_BASIS_JOIN); }
    ~Join() { (void)now(); }
  } join{st, aux, basis_started};
  HeadState* state = (HeadState*)(ws + w.head_state);
  float* basis = (float*)(ws + w.basis);
  float* gram_part = (float*)(ws + w.gram_part);
  float* mats = (float*)(ws + w.mats);
  float* delta = (float*)(ws + w.delta);
  static std::mutex attr_mu;
  static uint64_t attr_seen = 0;
  once_per_device(attr_mu, attr_seen, [] {
    (void)hipFuncSetAttribute((const void*)k_bf_keep_basis<T>, hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 128 * 8);
    (void)hipFuncSetAttribute((const void*)k_bf_keep_gram_part<T>, hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 128 * 8);
    (void)hipFuncSetAttribute((const void*)k_bf_finalize<T>, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * 128 * 129 * 4);
    (void)hipFuncSetAttribute((const void*)k_bf_lead<T>, hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)sizeof(float) * (128 * 129 + 4 + tri_work_floats(128, TE_MAXK) + TE_MAXK * 128));
  });
  if (var.subspace_iters > 0 && !(var.flags & VF_NAIVE) &&
      (rank > TE_MAXK || (var.flags & (VF_SUBSPACE_ALL | VF_SUBSPACE_EVR)) || m.d > 128)) {
    set_error("backfill: the subspace iteration takes the rank rule with pca_rank <= 16 and head_dim <= 128");
    return OBF_ERR_UNSUPPORTED;
  }
  if ((var.flags & VF_PER_TOKEN) &&
      (rank > TE_MAXK || (var.flags & (VF_SUBSPACE_ALL | VF_SUBSPACE_EVR | VF_NAIVE | VF_ATTN_INJECT)) || m.d > 128)) {
    set_error("backfill: the per-token variant takes the rank rule with pca_rank <= 16 and head_dim <= 128, without Naive Aggregation or Attn-inject");
    return OBF_ERR_UNSUPPORTED;
  }
  void* V_inject = (var.flags & VF_PER_TOKEN) ? nullptr : V_out;   // Per-token: the per-slot directions are added by a later kernel
  if (var.skips_basis()) {
    if (basis_started) { set_error("backfill: a basis was started for a variant without one"); return OBF_ERR_INVALID_ARG; }
    ProfScope prof_(ST_KEEP_BASIS, st);
    hipLaunchKernelGGL(k_bf_plain_state, dim3(m.heads), dim3(KB_THREADS), 0, st, scores, idx, n_keep, m.N, max_budget, rank, state, m.scs);
    if (check_launch("backfill plain state") != OBF_OK) return OBF_ERR_HIP;
  } else if (!basis_started) {
    // the caller did not start the bases earlier: try here (beside the statistics pass only)
    const obf_status_t bs = launch_backfill_basis(m, w, ws, V, scores, idx, n_keep, max_budget, rank, st, aux, &basis_started);
    join.armed = basis_started;
    if (bs != OBF_OK) return OBF_ERR_HIP;
  }
  if (!basis_started && !var.skips_basis()) {
    const size_t smem_kb = sizeof(double) * (size_t)m.d * m.d;
    int32_t* decided = nullptr;
    if (keep_cert_supported(m)) {
      decided = (int32_t*)(ws + w.decided);
      if (launch_keep_cert(m, V_out, 0, scores, idx, n_keep, max_budget, rank, state, decided, st, fro_part, diag != nullptr) != OBF_OK)
        return OBF_ERR_HIP;
    }
    ProfScope prof_(ST_KEEP_BASIS, st);
    // heads with at most d retained rows (none when the caller states that every budget is above d)
    if (!(min_budget > m.d && m.N > m.d) &&
        launch_keep_basis_small(m, V, scores, idx, n_keep, max_budget, rank, state, basis, st) != OBF_OK) return OBF_ERR_HIP;
    if (max_budget > m.d) {
      double* gpart = nullptr;
      if (max_budget >= kKeepGramMinBudget) {
        gpart = (double*)(ws + w.keep_gram);
        hipLaunchKernelGGL(k_bf_keep_gram_part<T>, dim3(kKeepGramChunks, kKeepGramSlots), dim3(KB_THREADS), smem_kb, st,
                           (const T*)V, idx, n_keep, decided, m.heads, m.N, m.d, max_budget, rank, m.kvs, gpart);
        if (check_launch("backfill keep_gram_part") != OBF_OK) return OBF_ERR_HIP;
      }
      hipLaunchKernelGGL(k_bf_keep_basis<T>, dim3(m.heads), dim3(KB_THREADS), smem_kb, st, (const T*)V, scores, idx, n_keep,
                         m.N, m.d, max_budget, rank, state, basis, decided, m.scs, m.kvs, gpart);
      if (check_launch("backfill keep_basis") != OBF_OK) return OBF_ERR_HIP;
    }
  }
  // while the bases are still being written on the second stream the statistics pass must not read the head states
  const int32_t* nk_stats = basis_started ? n_keep : nullptr;
  if (rank > 0 && del_stats_mfma_supported(m)) {
    // every budget above head_dim: the certificate settles nearly every head, the few others are found on the device
    const bool few_active = min_budget > m.d && m.N > m.d && !var.skips_basis();
    if (launch_del_stats_mfma(m, w, V, scores, idx, max_budget, state, nk_stats, gram_part, st, few_active) != OBF_OK) return OBF_ERR_HIP;
  } else if (rank > 0) {
    { ProfScope prof_(ST_DEL_STATS, st); hipLaunchKernelGGL(k_bf_del_stats<T>, dim3(w.nstat, m.heads), dim3(DS_THREADS), sizeof(float) * DS_TOK * m.d, st,
                       (const T*)V, scores, idx, m.N, m.d, max_budget, w.nstat, state, nk_stats, gram_part, m.scs, m.kvs); }
    if (check_launch("backfill del_stats") != OBF_OK) return OBF_ERR_HIP;
  }
  if (join.now() != OBF_OK) return OBF_ERR_HIP;
  {
    ProfScope prof_(ST_FINALIZE, st);
    const size_t one = sizeof(float) * m.d * (m.d + 1);
    // Heads that only need a few leading eigenpairs of a wide enough complement go to k_bf_lead after the finalisation
    // (not under the Max-P / EVR rules, which need the whole spectrum).  Its LDS is sized for complements up to 3d/4 wide
    // (two workgroups per CU); without the projection every complement is all of R^d, and it is sized for that.
    // The fast path of App. H lives in that kernel too and then takes every head that reaches Eq. 4.
    // So does the Per-token alternative (it needs the subspace itself, which only that kernel exports).
    const int iters = (var.flags & VF_NAIVE) ? 0 : var.subspace_iters;
    const bool all_lead = iters > 0 || (var.flags & VF_PER_TOKEN);
    const bool lead_ok = rank > 0 && rank <= TE_MAXK && !(var.flags & (VF_SUBSPACE_ALL | VF_SUBSPACE_EVR | VF_NAIVE)) &&
                         (all_lead || !(min_budget > m.d && m.N > m.d && !var.skips_basis()));
    LeadJob* lead = lead_ok ? (LeadJob*)(ws + w.lead_job) : (LeadJob*)nullptr;
    const int m_direct_max = ((var.flags & VF_NO_PROJECTION) || all_lead) ? m.d : 3 * m.d / 4;
    const int m_direct_min = all_lead ? 1 : FN_DIRECT_MIN;
    // every budget above head_dim: heads that need the finalisation are rare (the certificate settles the others), so one
    // launch with the large LDS size serves both classes instead of two launches that mostly exit at once
    const bool single = min_budget > m.d && m.N > m.d && !var.skips_basis();
    for (int cls = single ? -1 : 0; cls < (single ? 0 : 2); ++cls) {
      const size_t lds = (cls == 0) ? sizeof(float) * (size_t)fn_small_floats(m.d) : 2 * one;
      hipLaunchKernelGGL(k_bf_finalize<T>, dim3(m.heads), dim3(FN_THREADS), lds, st, m.N, m.d,
                         w.nstat, rank, state, basis, gram_part, mats, delta, delta_out, diag,
                         (rank > 0 && max_budget > 0) ? (T*)V_inject : (T*)nullptr, max_budget, cls, scores, idx,
                         var.flags, var.evr_tau, m.scs, (max_budget < m.d && rank > 0) ? (float*)(ws + w.rot) : (float*)nullptr,
                         lead, m_direct_min, m_direct_max);
    }
    if (check_launch("backfill finalize") != OBF_OK) return OBF_ERR_HIP;
    if (lead) {
      const int kq = rank < TE_MAXK ? rank : TE_MAXK;
      const size_t lds = sizeof(float) * ((size_t)m_direct_max * (m_direct_max | 1) + 4 + tri_work_floats(m_direct_max, kq) +
                                          (iters > 0 ? (size_t)kq * m.d : 0));
      hipLaunchKernelGGL(k_bf_lead<T>, dim3(m.heads), dim3(TE_THREADS), lds, st, m.d, rank, state, mats, delta, delta_out, diag,
                         (rank > 0 && max_budget > 0) ? (T*)V_inject : (T*)nullptr, max_budget, scores, idx, var.flags, m.scs,
                         (const LeadJob*)lead, iters);
      if (check_launch("backfill leading eigenpairs") != OBF_OK) return OBF_ERR_HIP;
    }
  }
  return OBF_OK;
}

obf_status_t launch_backfill(const Dims& m, const Workspace& w, char* ws, const void* V, const float* scores,
                             const int32_t* idx, const int32_t* n_keep, int32_t max_budget, int32_t rank,
                             void* V_out, float* delta_out, obf_diag_t* diag, hipStream_t st, hipStream_t aux,
                             const double* fro_part, bool basis_started, int32_t min_budget, Variant var) {
  if (m.dtype == OBF_BF16)
    return run<uint16_t>(m, w, ws, V, scores, idx, n_keep, max_budget, rank, V_out, delta_out, diag, st, aux, fro_part, basis_started, min_budget, var);
  return run<float>(m, w, ws, V, scores, idx, n_keep, max_budget, rank, V_out, delta_out, diag, st, aux, fro_part, basis_started, min_budget, var);
}

}  // namespace obf
