// Attention-mass scores (Eq. 1) on the matrix cores: bf16 operands, fp32 accumulation
// (v_mfma_f32_32x32x16_bf16), head_dim 128.
//
// A column sum of softmax rows needs every row's normaliser before any column can be summed, so
// K is streamed twice: pass A gives each query row's (max, sum-exp) over a chunk of tokens, a
// small kernel folds the chunks into log-sum-exp, pass B recomputes the logits and sums
// exp(logit - lse[row]) over the rows.  Both passes use the same register fragments of Q and K:
// an MFMA operand fragment holds, for lane l, 8 consecutive head_dim entries (l/32)*8.. of
// row l%32, for either operand, so swapping the two operands transposes the 32x32 output tile.
//   pass A computes (tokens x query rows): a lane then owns ONE query row per row block, and the
//          running (max, sum) needs two registers per row block;
//   pass B computes (query rows x tokens): a lane owns ONE token, and the column sum is an
//          in-lane sum plus one cross-lane add.
// The whole Q operand of a 128-row group lives in registers for the lifetime of a workgroup;
// K fragments are loaded straight from global memory in 16-byte pieces, one tile ahead.
#include "common.hpp"

namespace obf {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int SM_THREADS = 256;
constexpr int SM_WAVES = 4;
constexpr int SM_RB = 4;                 // 32-row blocks per row group
constexpr int SM_ROWS = SM_RB * 32;      // query rows per workgroup
constexpr int SM_D = 128;
constexpr int SM_KK = SM_D / 16;         // MFMA k-steps
constexpr int SM_TILE = 32;              // tokens per MFMA tile
constexpr float kLog2e = 1.4426950408889634f;

union Frag { uint4 u; bf16x8 v; };

__device__ __forceinline__ void load_q(Frag (&qf)[SM_RB][SM_KK], const uint16_t* __restrict__ Qh, int row0, int R, int lane) {
  const int r = lane & 31, kh = (lane >> 5) * 8;
#pragma unroll
  for (int rb = 0; rb < SM_RB; ++rb) {
    const int row = row0 + rb * 32 + r;
#pragma unroll
    for (int kk = 0; kk < SM_KK; ++kk) {
      if (row < R) qf[rb][kk].u = *(const uint4*)(Qh + (size_t)row * SM_D + kk * 16 + kh);
      else qf[rb][kk].u = make_uint4(0, 0, 0, 0);
    }
  }
}

__device__ __forceinline__ void load_k(Frag (&kf)[SM_KK], const uint16_t* __restrict__ Kh, int tok0, int t_end, int lane) {
  const int t = tok0 + (lane & 31), kh = (lane >> 5) * 8;
  if (t < t_end) {
    const uint4* p = (const uint4*)(Kh + (size_t)t * SM_D + kh);
#pragma unroll
    for (int kk = 0; kk < SM_KK; ++kk) kf[kk].u = p[kk * 2];
  } else {
#pragma unroll
    for (int kk = 0; kk < SM_KK; ++kk) kf[kk].u = make_uint4(0, 0, 0, 0);
  }
}

// ------------------------------------------------------------------------------------------------
// Pass A.  grid (nchunk * RG, heads); workgroup = 4 waves, each takes every 4th 32-token tile.
__global__ __launch_bounds__(SM_THREADS, 1) void k_score_stats_mfma(const uint16_t* __restrict__ K,
                                                                    const uint16_t* __restrict__ Q,
                                                                    double* __restrict__ stats_part, int N, int R,
                                                                    int nchunk, int RG) {
  __shared__ double s_m[SM_WAVES][SM_ROWS], s_l[SM_WAVES][SM_ROWS];
  const int head = blockIdx.y;
  const int chunk = blockIdx.x / RG, rg = blockIdx.x - chunk * RG;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t0 = chunk * kScoreChunk, t1 = min(N, t0 + kScoreChunk);
  const uint16_t* Kh = K + (size_t)head * N * SM_D;
  const uint16_t* Qh = Q + (size_t)head * R * SM_D;
  const int row0 = rg * SM_ROWS;
  const float a2 = kLog2e / sqrtf((float)SM_D);

  Frag qf[SM_RB][SM_KK];
  load_q(qf, Qh, row0, R, lane);
  float m[SM_RB];
  double l[SM_RB];
#pragma unroll
  for (int rb = 0; rb < SM_RB; ++rb) { m[rb] = -INFINITY; l[rb] = 0.0; }

  Frag kf[SM_KK], kn[SM_KK];
  int tok = t0 + wave * SM_TILE;
  if (tok < t1) load_k(kf, Kh, tok, t1, lane);
  for (; tok < t1; tok += SM_WAVES * SM_TILE) {
    const int nxt = tok + SM_WAVES * SM_TILE;
    if (nxt < t1) load_k(kn, Kh, nxt, t1, lane);
    f32x16 acc[SM_RB];
#pragma unroll
    for (int rb = 0; rb < SM_RB; ++rb) {
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rb][i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < SM_KK; ++kk)
        acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk].v, qf[rb][kk].v, acc[rb], 0, 0, 0);
    }
    // acc[rb][i]: token tok + (i/4)*8 + (lane/32)*4 + (i%4), query row row0 + rb*32 + lane%32
    const bool ragged = tok + SM_TILE > t1;
#pragma unroll
    for (int rb = 0; rb < SM_RB; ++rb) {
      float tv[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        tv[i] = acc[rb][i] * a2;
        if (ragged) {
          const int t = tok + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
          if (t >= t1) tv[i] = -INFINITY;
        }
      }
      float mx = tv[0];
#pragma unroll
      for (int i = 1; i < 16; ++i) mx = fmaxf(mx, tv[i]);
      const float mo = m[rb];
      const float mn = fmaxf(mo, mx);
      if (mn > -INFINITY) {
        float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
        for (int i = 0; i < 16; i += 4) {
          s0 += exp2f(tv[i] - mn); s1 += exp2f(tv[i + 1] - mn); s2 += exp2f(tv[i + 2] - mn); s3 += exp2f(tv[i + 3] - mn);
        }
        const float ts = (s0 + s1) + (s2 + s3);
        const double scale = (mo == mn) ? 1.0 : (double)exp2f(mo - mn);
        l[rb] = l[rb] * scale + (double)ts;
        m[rb] = mn;
      }
    }
    if (nxt < t1) {
#pragma unroll
      for (int kk = 0; kk < SM_KK; ++kk) kf[kk] = kn[kk];
    }
  }
  // fold the two lane halves (same query row, different tokens), then the four waves
#pragma unroll
  for (int rb = 0; rb < SM_RB; ++rb) {
    const float mo = __shfl_xor(m[rb], 32);
    const double lo = __shfl_xor(l[rb], 32);
    const float mn = fmaxf(m[rb], mo);
    double a = 0.0, b = 0.0;
    if (m[rb] > -INFINITY) a = l[rb] * exp2((double)(m[rb] - mn));
    if (mo > -INFINITY) b = lo * exp2((double)(mo - mn));
    // both halves compute the same sum in the same operand order: a is always the lower half's term
    const double sum = (lane < 32) ? (a + b) : (b + a);
    if (lane < 32) { s_m[wave][rb * 32 + lane] = (double)mn; s_l[wave][rb * 32 + lane] = sum; }
  }
  __syncthreads();
  if (threadIdx.x < SM_ROWS) {
    const int row = row0 + threadIdx.x;
    if (row < R) {
      double M = -INFINITY;
      for (int w = 0; w < SM_WAVES; ++w) M = fmax(M, s_m[w][threadIdx.x]);
      double L = 0.0;
      for (int w = 0; w < SM_WAVES; ++w)
        if (s_m[w][threadIdx.x] > -INFINITY) L += s_l[w][threadIdx.x] * exp2(s_m[w][threadIdx.x] - M);
      double* o = stats_part + (((size_t)head * nchunk + chunk) * R + row) * 2;
      o[0] = M * 0.6931471805599453;     // log2 units -> natural log, as the fold kernel expects
      o[1] = L;
    }
  }
}

// log-sum-exp of every query row from the chunk partials (same as the reference-precision path)
__global__ void k_score_lse_mfma(const double* __restrict__ stats_part, double* __restrict__ row_lse, int R, int nchunk,
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

// ------------------------------------------------------------------------------------------------
// Pass B.  Same grid.  out = scores (RG == 1) or the row group's partial column sums.
__global__ __launch_bounds__(SM_THREADS, 1) void k_score_mass_mfma(const uint16_t* __restrict__ K,
                                                                   const uint16_t* __restrict__ Q,
                                                                   const double* __restrict__ row_lse,
                                                                   float* __restrict__ out, int N, int R, int RG,
                                                                   size_t rg_stride) {
  const int head = blockIdx.y;
  const int chunk = blockIdx.x / RG, rg = blockIdx.x - chunk * RG;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t0 = chunk * kScoreChunk, t1 = min(N, t0 + kScoreChunk);
  const uint16_t* Kh = K + (size_t)head * N * SM_D;
  const uint16_t* Qh = Q + (size_t)head * R * SM_D;
  const double* lse = row_lse + (size_t)head * R;
  float* dst = out + (size_t)rg * rg_stride + (size_t)head * N;
  const int row0 = rg * SM_ROWS;
  const float a2 = kLog2e / sqrtf((float)SM_D);

  Frag qf[SM_RB][SM_KK];
  load_q(qf, Qh, row0, R, lane);
  // per-lane row offsets: row of acc[rb][i] is row0 + rb*32 + (i/4)*8 + (lane/32)*4 + (i%4)
  float b2[SM_RB][16];
#pragma unroll
  for (int rb = 0; rb < SM_RB; ++rb)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int row = row0 + rb * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
      b2[rb][i] = (row < R) ? (float)(lse[row] * 1.4426950408889634) : INFINITY;   // padded rows contribute exp2(-inf) = 0
    }

  Frag kf[SM_KK], kn[SM_KK];
  int tok = t0 + wave * SM_TILE;
  if (tok < t1) load_k(kf, Kh, tok, t1, lane);
  for (; tok < t1; tok += SM_WAVES * SM_TILE) {
    const int nxt = tok + SM_WAVES * SM_TILE;
    if (nxt < t1) load_k(kn, Kh, nxt, t1, lane);
    f32x16 acc[SM_RB];
#pragma unroll
    for (int rb = 0; rb < SM_RB; ++rb) {
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rb][i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < SM_KK; ++kk)
        acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[rb][kk].v, kf[kk].v, acc[rb], 0, 0, 0);
    }
    float c0 = 0.f, c1 = 0.f, c2 = 0.f, c3 = 0.f;
#pragma unroll
    for (int rb = 0; rb < SM_RB; ++rb) {
#pragma unroll
      for (int i = 0; i < 16; i += 4) {
        c0 += exp2f(fmaf(acc[rb][i], a2, -b2[rb][i]));
        c1 += exp2f(fmaf(acc[rb][i + 1], a2, -b2[rb][i + 1]));
        c2 += exp2f(fmaf(acc[rb][i + 2], a2, -b2[rb][i + 2]));
        c3 += exp2f(fmaf(acc[rb][i + 3], a2, -b2[rb][i + 3]));
      }
    }
    float col = (c0 + c1) + (c2 + c3);
    const float other = __shfl_xor(col, 32);
    col = (lane < 32) ? (col + other) : (other + col);
    const int t = tok + (lane & 31);
    if (lane < 32 && t < t1) dst[t] = col;
    if (nxt < t1) {
#pragma unroll
      for (int kk = 0; kk < SM_KK; ++kk) kf[kk] = kn[kk];
    }
  }
}

// scores = sum of the row groups' partial column sums (fixed order)
__global__ void k_score_sum_groups(const float* __restrict__ part, float* __restrict__ scores, size_t n, int RG,
                                   size_t rg_stride) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float s = 0.f;
  for (int g = 0; g < RG; ++g) s += part[(size_t)g * rg_stride + i];
  scores[i] = s;
}

bool mfma_score_supported(const Dims& m) {
  return m.dtype == OBF_BF16 && m.d == SM_D;
}

obf_status_t launch_score_mfma(const Dims& m, const Workspace& w, char* ws, const void* K, const void* Q,
                               float* scores, double* row_lse, hipStream_t st) {
  double* stats_part = (double*)(ws + w.stats_part);
  const int RG = (m.R + SM_ROWS - 1) / SM_ROWS;
  const size_t rg_stride = (size_t)m.heads * m.N;
  float* part = (RG > 1) ? (float*)(ws + w.score_part) : scores;
  dim3 grid(w.nchunk * RG, m.heads);
  { ProfScope prof_(ST_SCORE_STATS, st);
    hipLaunchKernelGGL(k_score_stats_mfma, grid, dim3(SM_THREADS), 0, st, (const uint16_t*)K, (const uint16_t*)Q,
                       stats_part, m.N, m.R, w.nchunk, RG); }
  if (check_launch("score stats (mfma)") != OBF_OK) return OBF_ERR_HIP;
  const int total_rows = m.heads * m.R;
  { ProfScope prof_(ST_SCORE_LSE, st);
    hipLaunchKernelGGL(k_score_lse_mfma, dim3((total_rows + 255) / 256), dim3(256), 0, st, stats_part, row_lse, m.R,
                       w.nchunk, total_rows); }
  if (check_launch("score lse (mfma)") != OBF_OK) return OBF_ERR_HIP;
  { ProfScope prof_(ST_SCORE_MASS, st);
    hipLaunchKernelGGL(k_score_mass_mfma, grid, dim3(SM_THREADS), 0, st, (const uint16_t*)K, (const uint16_t*)Q, row_lse,
                       part, m.N, m.R, RG, rg_stride); }
  if (check_launch("score mass (mfma)") != OBF_OK) return OBF_ERR_HIP;
  if (RG > 1) {
    const size_t n = (size_t)m.heads * m.N;
    hipLaunchKernelGGL(k_score_sum_groups, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, part, scores, n, RG,
                       rg_stride);
    if (check_launch("score sum groups") != OBF_OK) return OBF_ERR_HIP;
  }
  return OBF_OK;
}

}  // namespace obf
