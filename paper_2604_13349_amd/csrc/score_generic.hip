// Attention-mass scores (Eq. 1), reference-precision path: every logit, exponential and sum is
// carried in double on the vector ALU.  Used for fp32 I/O and for shapes the MFMA path does not
// take.  Two passes over K because a column sum of softmax rows needs every row's normaliser
// first: pass A gives per-row log-sum-exp, pass B the column sums.
#include "common.hpp"

namespace obf {

constexpr int GS_ROWS = 32;     // query rows per tile
constexpr int GS_TOK = 64;      // tokens per tile
constexpr int GS_THREADS = 256;

template <typename T>
__device__ __forceinline__ void load_tile(float* dst, int ld, const T* src, int rows_valid, int rows_total, int d) {
  // dst[r][c] = src[r*d + c] for r < rows_valid, zero otherwise
  for (int e = threadIdx.x; e < rows_total * d; e += GS_THREADS) {
    int r = e / d, c = e - r * d;
    dst[r * ld + c] = (r < rows_valid) ? Elem<T>::load(src + (size_t)r * d + c) : 0.0f;
  }
}

// Pass A: partial (max, sum exp(logit - max)) per query row over one chunk of tokens.
template <typename T>
__global__ __launch_bounds__(GS_THREADS) void k_score_stats_generic(const T* __restrict__ K, const T* __restrict__ Q,
                                                                    double* __restrict__ stats_part, int N, int d, int R,
                                                                    int nchunk, int chunk_tokens, int kvs) {
  extern __shared__ float smem[];
  const int ld = d + 1;
  float* Qs = smem;                   // [GS_ROWS][ld]
  float* Ks = smem + GS_ROWS * ld;    // [GS_TOK][ld]
  const int head = blockIdx.y, chunk = blockIdx.x;
  const int t0 = chunk * chunk_tokens;
  const int t1 = min(N, t0 + chunk_tokens);
  const T* Kh = K + (size_t)head * kvs * d;
  const T* Qh = Q + (size_t)head * R * d;
  const int rr = threadIdx.x >> 3, tl = threadIdx.x & 7;
  const double scale = 1.0 / sqrt((double)d);

  for (int r0 = 0; r0 < R; r0 += GS_ROWS) {
    __syncthreads();
    load_tile<T>(Qs, ld, Qh + (size_t)r0 * d, min(GS_ROWS, R - r0), GS_ROWS, d);
    double m = -INFINITY, l = 0.0;
    for (int tt = t0; tt < t1; tt += GS_TOK) {
      __syncthreads();
      const int tv = min(GS_TOK, t1 - tt);
      load_tile<T>(Ks, ld, Kh + (size_t)tt * d, tv, GS_TOK, d);
      __syncthreads();
      for (int i = 0; i < GS_TOK / 8; ++i) {
        const int t = tl + 8 * i;
        if (t < tv) {
          double acc = 0.0;
          const float* q = Qs + rr * ld;
          const float* k = Ks + t * ld;
          for (int c = 0; c < d; ++c) acc = fma((double)q[c], (double)k[c], acc);
          const double s = acc * scale;
          if (s > m) { l = l * exp(m - s) + 1.0; m = s; }
          else l += exp(s - m);
        }
      }
    }
    // combine the 8 token lanes of a row (consecutive lanes)
    for (int off = 1; off < 8; off <<= 1) {
      const double m2 = __shfl_xor(m, off), l2 = __shfl_xor(l, off);
      const double M = fmax(m, m2);
      const double a = (m == -INFINITY) ? 0.0 : l * exp(m - M);
      const double b = (m2 == -INFINITY) ? 0.0 : l2 * exp(m2 - M);
      m = M; l = a + b;
    }
    const int row = r0 + rr;
    if (tl == 0 && row < R) {
      double* o = stats_part + (((size_t)head * nchunk + chunk) * R + row) * 2;
      o[0] = m; o[1] = l;
    }
  }
}

// log-sum-exp of every query row from the chunk partials.
__global__ void k_score_lse(const double* __restrict__ stats_part, double* __restrict__ row_lse, int R, int nchunk,
                            int total_rows) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total_rows) return;
  const int head = i / R, row = i - head * R;
  double M = -INFINITY;
  for (int c = 0; c < nchunk; ++c) M = fmax(M, stats_part[(((size_t)head * nchunk + c) * R + row) * 2]);
  double L = 0.0;
  for (int c = 0; c < nchunk; ++c) {
    const double* p = stats_part + (((size_t)head * nchunk + c) * R + row) * 2;
    if (p[0] != -INFINITY) L += p[1] * exp(p[0] - M);
  }
  row_lse[i] = M + log(L);
}

// Pass B: scores[j] = sum_rows exp(logit - lse[row]).
template <typename T>
__global__ __launch_bounds__(GS_THREADS) void k_score_mass_generic(const T* __restrict__ K, const T* __restrict__ Q,
                                                                   const double* __restrict__ row_lse,
                                                                   float* __restrict__ scores, int N, int d, int R, int chunk_tokens, int kvs) {
  extern __shared__ float smem[];
  const int ld = d + 1;
  float* Qs = smem;
  float* Ks = smem + GS_ROWS * ld;
  double* red = (double*)(smem + (GS_ROWS + GS_TOK) * ld + ((GS_ROWS + GS_TOK) * ld & 1));   // [GS_ROWS][GS_TOK]
  const int head = blockIdx.y, chunk = blockIdx.x;
  const int t0 = chunk * chunk_tokens;
  const int t1 = min(N, t0 + chunk_tokens);
  const T* Kh = K + (size_t)head * kvs * d;
  const T* Qh = Q + (size_t)head * R * d;
  const double* lse = row_lse + (size_t)head * R;
  const int rr = threadIdx.x >> 3, tl = threadIdx.x & 7;
  const double scale = 1.0 / sqrt((double)d);

  for (int tt = t0; tt < t1; tt += GS_TOK) {
    const int tv = min(GS_TOK, t1 - tt);
    __syncthreads();
    load_tile<T>(Ks, ld, Kh + (size_t)tt * d, tv, GS_TOK, d);
    double col[GS_TOK / 8];
    for (int i = 0; i < GS_TOK / 8; ++i) col[i] = 0.0;
    for (int r0 = 0; r0 < R; r0 += GS_ROWS) {
      __syncthreads();
      load_tile<T>(Qs, ld, Qh + (size_t)r0 * d, min(GS_ROWS, R - r0), GS_ROWS, d);
      __syncthreads();
      const int row = r0 + rr;
      if (row < R) {
        const double L = lse[row];
        const float* q = Qs + rr * ld;
        for (int i = 0; i < GS_TOK / 8; ++i) {
          const int t = tl + 8 * i;
          if (t < tv) {
            double acc = 0.0;
            const float* k = Ks + t * ld;
            for (int c = 0; c < d; ++c) acc = fma((double)q[c], (double)k[c], acc);
            col[i] += exp(acc * scale - L);
          }
        }
      }
    }
    for (int i = 0; i < GS_TOK / 8; ++i) red[rr * GS_TOK + tl + 8 * i] = col[i];
    __syncthreads();
    if (threadIdx.x < tv) {
      double s = 0.0;
      for (int r = 0; r < GS_ROWS; ++r) s += red[r * GS_TOK + threadIdx.x];
      scores[(size_t)head * N + tt + threadIdx.x] = (float)s;
    }
  }
}

template <typename T>
static obf_status_t run(const Dims& m, const Workspace& w, char* ws, const void* K, const void* Q, float* scores,
                        double* row_lse, hipStream_t st) {
  double* stats_part = (double*)(ws + w.stats_part);
  const size_t ld = m.d + 1;
  const size_t smemA = sizeof(float) * (GS_ROWS + GS_TOK) * ld;
  const size_t smemB = smemA + 8 + sizeof(double) * GS_ROWS * GS_TOK;
  dim3 grid(w.nchunk, m.heads);
  { ProfScope prof_(ST_SCORE_STATS, st); hipLaunchKernelGGL(k_score_stats_generic<T>, grid, dim3(GS_THREADS), smemA, st, (const T*)K, (const T*)Q, stats_part,
                     m.N, m.d, m.R, w.nchunk, w.chunk_tokens, m.kvs); }
  if (check_launch("score stats (generic)") != OBF_OK) return OBF_ERR_HIP;
  const int total_rows = m.heads * m.R;
  { ProfScope prof_(ST_SCORE_LSE, st); hipLaunchKernelGGL(k_score_lse, dim3((total_rows + 255) / 256), dim3(256), 0, st, stats_part, row_lse, m.R, w.nchunk,
                     total_rows); }
  if (check_launch("score lse") != OBF_OK) return OBF_ERR_HIP;
  { ProfScope prof_(ST_SCORE_MASS, st); hipLaunchKernelGGL(k_score_mass_generic<T>, grid, dim3(GS_THREADS), smemB, st, (const T*)K, (const T*)Q, row_lse, scores,
                     m.N, m.d, m.R, w.chunk_tokens, m.kvs); }
  return check_launch("score mass (generic)");
}

obf_status_t launch_score_generic(const Dims& m, const Workspace& w, char* ws, const void* K, const void* Q,
                                  float* scores, double* row_lse, hipStream_t st) {
  if (m.dtype == OBF_BF16) return run<uint16_t>(m, w, ws, K, Q, scores, row_lse, st);
  return run<float>(m, w, ws, K, Q, scores, row_lse, st);
}

}  // namespace obf
