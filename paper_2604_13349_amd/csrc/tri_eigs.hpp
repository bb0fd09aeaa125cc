// Leading eigenpairs of a small symmetric matrix, for a workgroup of 512 threads: the direct route for
// the case "a few leading right singular vectors of the residual" (Sec. 4.4: k = pca_rank is small against the
// width of the complement), in place of a full Jacobi diagonalisation:
//   1. Householder tridiagonalisation T = H S H^T (m - 2 reflectors, four barriers each);
//   2. the k largest eigenvalues of the tridiagonal S by multisection on Sturm counts (every thread evaluates one
//      shift per round; three or four rounds shrink an eigenvalue's bracket below single-precision resolution);
//   3. their eigenvectors by inverse iteration on S - theta I (tridiagonal elimination with row exchanges, one lane
//      per eigenvector, three solves from a fixed pseudo-random start), eight at a time;
//   4. back-transformation through the reflectors (one wave per eigenvector) and a final Gram-Schmidt pass over the
//      k vectors (eigenvalues that agree to rounding give vectors that only span the right subspace together).
// All arithmetic is single precision; nothing here depends on convergence of an iteration.
#pragma once
#include "common.hpp"
#include "wave_ops.hpp"

namespace obf {

constexpr int TE_THREADS = 512;
constexpr int TE_WAVES = TE_THREADS / 64;
constexpr int TE_MAXK = 16;              // most eigenpairs
constexpr int TE_BATCH = 8;              // eigenvectors per pass of the inverse iteration and the back-transformation (one wave each)
constexpr int TE_CPT = 32;               // columns per thread of the register-resident matrix (128 rows x 4 groups)

// floats of LDS scratch tri_top_eigs needs for an m x m matrix and k eigenpairs
__host__ __device__ inline int tri_lane_stride(int k) { return k <= 4 ? 4 : 8; }
__host__ __device__ inline int tri_work_floats(int m, int k) {
  return 4 * m + 256 + TE_THREADS + 96 + 7 * tri_lane_stride(k) * m + (k > TE_BATCH ? k * m : 0);
}

// sum over the 64 lanes, the result in every lane: four in-row DPP steps, then the rows and the halves meet through
// lane swaps (no LDS traffic, a fixed order of additions)
__device__ __forceinline__ float te_wave_sum(float v) {
  v += __uint_as_float(OBF_DPP_MOV(__float_as_uint(v), 0xB1));
  v += __uint_as_float(OBF_DPP_MOV(__float_as_uint(v), 0x4E));
  v += __uint_as_float(OBF_DPP_MOV(__float_as_uint(v), 0x141));
  v += __uint_as_float(OBF_DPP_MOV(__float_as_uint(v), 0x140));
  const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// Inverse iteration on the tridiagonal S - theta I for one eigenvector per lane.  Arrays of the factorisation live at
// f[(q * m + j) * KS] for q = 0 .. 4: the upper triangle's three diagonals (the first as its reciprocal), the
// multiplier and the row-exchange flag of step j (elimination with partial pivoting).  KS, the lane stride, is a
// compile-time constant so that the compiler can tell the entries apart and keep the loads ahead of the stores.
template <int KS>
__device__ __forceinline__ void te_factor(const float* __restrict__ dv, const float* __restrict__ ev, const int m,
                                          const float theta, const float tiny, float* __restrict__ f) {
  float* i0 = f; float* a1 = f + m * KS; float* a2 = a1 + m * KS; float* mu = a2 + m * KS; float* sw = mu + m * KS;
  float r0 = dv[0] - theta, r1 = (m > 1) ? ev[0] : 0.f, r2 = 0.f;
#pragma unroll 4
  for (int j = 0; j + 1 < m; ++j) {
    float n0 = ev[j], n1 = dv[j + 1] - theta, n2 = (j + 2 < m) ? ev[j + 1] : 0.f;
    const bool swap = fabsf(n0) > fabsf(r0);
    if (swap) { float t; t = r0; r0 = n0; n0 = t; t = r1; r1 = n1; n1 = t; t = r2; r2 = n2; n2 = t; }
    if (r0 == 0.f) r0 = tiny;
    float inv = __builtin_amdgcn_rcpf(r0);                      // one Newton step on the hardware reciprocal: the pivots only
    inv = fmaf(fmaf(-r0, inv, 1.f), inv, inv);                  // steer an iteration that converges whatever their last bit
    const float g = n0 * inv;
    i0[j * KS] = inv; a1[j * KS] = r1; a2[j * KS] = r2; mu[j * KS] = g; sw[j * KS] = swap ? 1.f : 0.f;
    r0 = fmaf(-g, r1, n1); r1 = fmaf(-g, r2, n2); r2 = 0.f;
  }
  i0[(m - 1) * KS] = 1.f / ((fabsf(r0) > 1e-3f * tiny) ? r0 : tiny);
  a1[(m - 1) * KS] = 0.f; a2[(m - 1) * KS] = 0.f;
}

// the row operations of the elimination applied to the right-hand side: scale * in -> out
template <int KS>
__device__ __forceinline__ void te_forward(const float* __restrict__ f, const int m, const float* __restrict__ in,
                                           float* __restrict__ out, const float scale) {
  const float* mu = f + 3 * m * KS; const float* sw = mu + m * KS;
  float carry = in[0] * scale;
#pragma unroll 4
  for (int j = 0; j + 1 < m; ++j) {
    const float nx = in[(j + 1) * KS] * scale, g = mu[j * KS];
    const bool swap = sw[j * KS] != 0.f;
    const float bj = swap ? nx : carry, bn = swap ? carry : nx;
    out[j * KS] = bj;
    carry = fmaf(-g, bj, bn);
  }
  out[(m - 1) * KS] = carry;
}

// back substitution with the upper triangle: in -> out; returns the largest magnitude of the solution
template <int KS>
__device__ __forceinline__ float te_backward(const float* __restrict__ f, const int m, const float* __restrict__ in,
                                             float* __restrict__ out) {
  const float* i0 = f; const float* a1 = f + m * KS; const float* a2 = a1 + m * KS;
  float z1 = 0.f, z2 = 0.f, big = 0.f;
#pragma unroll 4
  for (int j = m - 1; j >= 0; --j) {
    const float v = (in[j * KS] - a1[j * KS] * z1 - a2[j * KS] * z2) * i0[j * KS];
    out[j * KS] = v;
    z2 = z1; z1 = v;
    big = fmaxf(big, fabsf(v));
  }
  return big;
}

// Tsrc: the m x m symmetric matrix (row stride ls; global or LDS, read once).  Rf: LDS, m rows of stride lt (odd), receives
// the reflectors (column j below the sub-diagonal).  m <= 128.
// work: LDS scratch of tri_work_floats(m, k) floats, 16-byte aligned.  1 <= k <= min(m, TE_MAXK); KS = tri_lane_stride(k).
// More than TE_BATCH eigenpairs are found in passes of TE_BATCH (the eigenvalues' multisection, the inverse iteration and
// the back-transformation each run once per pass on the same scratch).
// On return (after its own final barrier) *theta points at the k eigenvalues, largest first, and *W at the k unit
// eigenvectors, W[i * m + t].  Every thread of the workgroup must call.
template <int KS>
__device__ __forceinline__ void tri_top_eigs(const float* __restrict__ Tsrc, const int ls, float* Rf, const int lt, const int m,
                                             const int k, float* work, const float** theta, const float** W) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  float* vv = work;                   // [128] reflector, zero outside the trailing block and past the matrix (work is 16-byte aligned)
  float* pv = vv + 128;               // [128] beta T v, likewise
  float* dv = pv + 128;               // diagonal of S
  float* ev = dv + m;                 // sub-diagonal of S: ev[j] = S[j+1][j]
  float* e2 = ev + m;
  float* bet = e2 + m;                // reflector j is I - bet[j] v v^T, v in column j of Rf
  int* cnt = (int*)(bet + m);         // [TE_THREADS]
  float* br_a = (float*)(cnt + TE_THREADS); // [16] brackets, then eigenvalues
  float* br_b = br_a + 16;
  float* th = br_b + 16;
  int* wc = (int*)(th + 16);          // [16] per-wave counts
  float* scal = (float*)(wc + 16);    // [32] lo, hi, ...
  float* lu = scal + 32;              // [5][m][KS] factors of S - theta I per eigenvector + [m][KS] second iteration vector; later W [k][m]
  float* zz = lu + 6 * m * KS;        // [m][KS] iteration vectors

  // ---- 1. tridiagonalisation.  The matrix lives in registers: thread (a, g) = (tid % 128, tid / 128) owns row a, columns
  // g, g + 4, ..., g + 124 (absolute numbering throughout; vv and pv are zero in front of the trailing block, so no
  // column needs masking).  The cyclic deal keeps the four column groups equally busy while the trailing block shrinks:
  // a group's columns come in four blocks of eight, and a block that lies in front of the trailing block (or past the
  // matrix) is skipped by the whole wave, as is a wave all of whose 64 rows do.  Per reflector: wave 0 forms v from the
  // column the owners published, all threads form their share of T v, the rows add the four shares, and the symmetric
  // rank-two update stays in registers.  LDS carries only vectors and receives the reflectors.
  const int ra = tid & 127;
  const int rg = __builtin_amdgcn_readfirstlane(tid >> 7);
  const int row_lo = (wave & 1) * 64;                          // the rows of this wave: row_lo .. row_lo + 63
  float* part = (float*)cnt;                                   // [4][128] shares of T v (the counts come later)
  float* xcol = e2;                                            // the published column (e2 is free until the form is complete)
  float tr[TE_CPT];
#pragma unroll
  for (int c = 0; c < TE_CPT; ++c)                              // symmetric: entry (ra, col) is read as (col, ra), lanes along a row
    tr[c] = (ra < m && rg + 4 * c < m) ? Tsrc[(size_t)(rg + 4 * c) * ls + ra] : 0.f;
  if (tid < 128) { vv[tid] = 0.f; pv[tid] = 0.f; }
  if (rg == 0 && ra < m) xcol[ra] = tr[0];                     // column 0
  if (tid == 0) dv[0] = tr[0];
  __syncthreads();
  // A wave's threads share their 32 columns (rg is the same for all of them): each lane fetches one entry of v and of
  // p, and the others' entries arrive as scalar operands through lane reads - no LDS broadcast traffic.
  const int cmine = rg + 4 * (lane & 31);
  auto lane_val = [](const float x, const int l) -> float {
    return __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(x), l));
  };
  for (int j = 0; j + 2 < m; ++j) {
    // wave 0 forms the reflector from the published column.  Single-instruction square root and reciprocal (1 ulp): the
    // reflector only has to be orthogonal to rounding.
    if (wave == 0) {
      const int i0 = j + 1 + lane, i1 = i0 + 64;               // absolute rows of the column below the diagonal
      const float x0 = (i0 < m) ? xcol[i0] : 0.f, x1 = (i1 < m) ? xcol[i1] : 0.f;
      const float sigma = __builtin_amdgcn_sqrtf(te_wave_sum(fmaf(x0, x0, x1 * x1)));
      const float head = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(x0)));
      const float alpha = (head >= 0.f) ? -sigma : sigma;
      const float v0 = (lane == 0) ? x0 - alpha : x0;
      if (i0 < m) { vv[i0] = v0; Rf[i0 * lt + j] = v0; }        // the reflector, kept for the back-transformation
      if (i1 < m) { vv[i1] = x1; Rf[i1 * lt + j] = x1; }
      if (lane == 0) {
        vv[j] = 0.f; pv[j] = 0.f;                              // row / column j have left the trailing block
        bet[j] = (sigma > 0.f) ? __builtin_amdgcn_rcpf(sigma * (sigma + fabsf(head))) : 0.f;
        ev[j] = (sigma > 0.f) ? alpha : 0.f;
      }
    }
    __syncthreads();
    const float beta = bet[j];
    const bool rows_live = row_lo + 63 > j && row_lo < m;      // uniform over the wave
    if (beta != 0.f) {                                         // uniform
      const float vmine = vv[cmine];
      if (rows_live) {
        float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;           // four independent chains
#pragma unroll
        for (int b = 0; b < TE_CPT / 8; ++b) {
          if (rg + 32 * b + 28 > j && rg + 32 * b < m) {        // uniform: the block reaches into the trailing block
#pragma unroll
            for (int c = 8 * b; c < 8 * b + 8; c += 4) {
              s0 = fmaf(tr[c], lane_val(vmine, c), s0); s1 = fmaf(tr[c + 1], lane_val(vmine, c + 1), s1);
              s2 = fmaf(tr[c + 2], lane_val(vmine, c + 2), s2); s3 = fmaf(tr[c + 3], lane_val(vmine, c + 3), s3);
            }
          }
        }
        if (ra > j && ra < m) part[rg * 128 + ra] = (s0 + s1) + (s2 + s3);
      }
      __syncthreads();
      if (tid > j && tid < m) pv[tid] = beta * ((part[tid] + part[128 + tid]) + (part[256 + tid] + part[384 + tid]));
      __syncthreads();
      const float K = 0.5f * beta * te_wave_sum(fmaf(pv[lane], vv[lane], pv[lane + 64] * vv[lane + 64]));   // the same in every wave
      if (rows_live) {
        // rows outside the trailing block (and past the matrix) have v = p = 0: their registers do not change
        const float va = vv[ra], wa = fmaf(-K, va, pv[ra]);
        const float wmine = fmaf(-K, vmine, pv[cmine]);      // w = p - K v of this lane's column
#pragma unroll
        for (int b = 0; b < TE_CPT / 8; ++b) {
          if (rg + 32 * b + 28 > j && rg + 32 * b < m) {
#pragma unroll
            for (int c = 8 * b; c < 8 * b + 8; ++c) tr[c] -= fmaf(va, lane_val(wmine, c), wa * lane_val(vmine, c));
          }
        }
      }
    }
    // the owners publish column j + 1 of the updated block (and its diagonal entry, final from here on); the column's
    // position in the register array is the same for the whole workgroup: a jump, not a chain of selects
    if (rg == ((j + 1) & 3) && ra > j && ra < m) {
      float xv = 0.f;
      switch ((j + 1) >> 2) {
#define OBF_TE_CASE(q) case q: xv = tr[q]; break;
        OBF_TE_CASE(0) OBF_TE_CASE(1) OBF_TE_CASE(2) OBF_TE_CASE(3) OBF_TE_CASE(4) OBF_TE_CASE(5) OBF_TE_CASE(6) OBF_TE_CASE(7)
        OBF_TE_CASE(8) OBF_TE_CASE(9) OBF_TE_CASE(10) OBF_TE_CASE(11) OBF_TE_CASE(12) OBF_TE_CASE(13) OBF_TE_CASE(14) OBF_TE_CASE(15)
        OBF_TE_CASE(16) OBF_TE_CASE(17) OBF_TE_CASE(18) OBF_TE_CASE(19) OBF_TE_CASE(20) OBF_TE_CASE(21) OBF_TE_CASE(22) OBF_TE_CASE(23)
        OBF_TE_CASE(24) OBF_TE_CASE(25) OBF_TE_CASE(26) OBF_TE_CASE(27) OBF_TE_CASE(28) OBF_TE_CASE(29) OBF_TE_CASE(30) OBF_TE_CASE(31)
#undef OBF_TE_CASE
        default: break;
      }
      xcol[ra] = xv;
      if (ra == j + 1) dv[j + 1] = xv;
    }
    __syncthreads();
  }
  // the last 2 x 2 block: its diagonal entries and the sub-diagonal entry between them
  if (m >= 2) {
    if (rg == ((m - 1) & 3) && ra == m - 1) {
      float xv = 0.f;
#pragma unroll
      for (int c = 0; c < TE_CPT; ++c) if (c == (m - 1) >> 2) xv = tr[c];
      dv[m - 1] = xv;
    }
    if (rg == ((m - 2) & 3) && ra == m - 1) {
      float xv = 0.f;
#pragma unroll
      for (int c = 0; c < TE_CPT; ++c) if (c == (m - 2) >> 2) xv = tr[c];
      ev[m - 2] = xv;
    }
  }
  __syncthreads();
  if (wave == 0) {
    // Gershgorin interval of S and its largest squared sub-diagonal entry: lane l looks at rows l and l + 64
    float lo = INFINITY, hi = -INFINITY, me2 = 0.f;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int i = lane + 64 * h;
      if (i < m) {
        const float below = (i + 1 < m) ? ev[i] : 0.f, above = (i > 0) ? ev[i - 1] : 0.f;
        const float r = fabsf(above) + fabsf(below);
        lo = fminf(lo, dv[i] - r); hi = fmaxf(hi, dv[i] + r);
        me2 = fmaxf(me2, below * below);
        e2[i] = below * below;
      }
    }
    for (int off = 32; off > 0; off >>= 1) {
      lo = fminf(lo, __shfl_xor(lo, off)); hi = fmaxf(hi, __shfl_xor(hi, off)); me2 = fmaxf(me2, __shfl_xor(me2, off));
    }
    if (lane == 0) {
      const float span = hi - lo;
      scal[0] = lo - (1e-3f * span + 1e-30f);
      scal[1] = hi + (1e-3f * span + 1e-30f);
      scal[2] = 1e-30f * fmaxf(1.f, me2);                        // smallest pivot magnitude of the Sturm recurrence
      scal[3] = 1.2e-7f * fmaxf(fabsf(lo), fabsf(hi));           // pivot perturbation of the inverse iteration
    }
  }
  __syncthreads();

  // ---- 2. eigenvalues: number of eigenvalues below x = number of negative terms of the Sturm recurrence
  const float pivmin = scal[2];
  auto sturm = [&](const float x) -> int {
    float q = dv[0] - x;
    int c = q < 0.f;
    for (int i = 1; i < m; ++i) {
      if (fabsf(q) < pivmin) q = (q < 0.f) ? -pivmin : pivmin;
      q = dv[i] - x - e2[i - 1] * __builtin_amdgcn_rcpf(q);
      c += q < 0.f;
    }
    return c;
  };
  {
    const float lo = scal[0], hi = scal[1];
    constexpr float step = 1.f / (float)(TE_THREADS + 1);
    cnt[tid] = sturm(lo + (hi - lo) * ((float)(tid + 1) * step));
    __syncthreads();
    if (tid < k) {                                             // eigenvalue tid from the top is number m - 1 - tid from below
      const int tgt = m - 1 - tid;
      int a = 0, b = TE_THREADS;                               // first shift whose count exceeds tgt
      while (a < b) { const int mid = (a + b) >> 1; if (cnt[mid] <= tgt) a = mid + 1; else b = mid; }
      br_a[tid] = (a > 0) ? lo + (hi - lo) * ((float)a * step) : lo;
      br_b[tid] = (a < TE_THREADS) ? lo + (hi - lo) * ((float)(a + 1) * step) : hi;
    }
    __syncthreads();
  }
  for (int g0 = 0; g0 < k; g0 += TE_BATCH) {                   // eigenvalues g0 .. g0 + kb - 1 (from the top)
    const int kb = min(TE_BATCH, k - g0);
    int kp = 1;
    while (kp < kb) kp <<= 1;
    const int S = TE_THREADS / kp;                             // shifts per eigenvalue and round (a multiple of 64)
    const int g = tid / S, s = tid - g * S;
    // round one left a bracket of 1/513 of the spectrum's extent; each further round divides it by S + 1: two rounds of
    // 257 reach 3e-8 of the extent, half a unit in the last place of the largest eigenvalue
    const int rounds = (2 * S >= TE_THREADS) ? 2 : 3;
    for (int round = 0; round < rounds; ++round) {
      bool below = false;
      float a = 0.f, b = 0.f;
      if (g < kb) {
        a = br_a[g0 + g]; b = br_b[g0 + g];
        below = sturm(a + (b - a) * ((float)(s + 1) / (float)(S + 1))) <= m - 1 - (g0 + g);
      }
      const int c = __popcll(__ballot(below));
      if (lane == 0) wc[wave] = c;
      __syncthreads();
      if (tid < kb) {
        const float a2 = br_a[g0 + tid], b2 = br_b[g0 + tid];
        int p = 0;
        for (int w = 0; w < S / 64; ++w) p += wc[tid * (S / 64) + w];
        // counts are monotone in the shift: the first p shifts are at or below the eigenvalue
        if (p > 0) br_a[g0 + tid] = a2 + (b2 - a2) * ((float)p / (float)(S + 1));
        if (p < S) br_b[g0 + tid] = a2 + (b2 - a2) * ((float)(p + 1) / (float)(S + 1));
      }
      __syncthreads();
    }
    if (tid < kb) th[g0 + tid] = 0.5f * (br_a[g0 + tid] + br_b[g0 + tid]);
    __syncthreads();
  }

  // ---- 3. eigenvectors of S: inverse iteration, lane i of wave 0 owns eigenvector b0 + i; 4. back-transformation
  // w = H_0 H_1 ... H_{m-3} z, one wave per eigenvector, lane l holds entries l and l + 64
  float* Wv = (k > TE_BATCH) ? zz + m * KS : lu;               // [k][m]; a single pass leaves it where the factors were
  for (int b0 = 0; b0 < k; b0 += TE_BATCH) {
    const int kb = min(TE_BATCH, k - b0);
    if (wave == 0 && lane < kb) {
      float* za = zz + lane;
      float* zb = lu + 5 * m * KS + lane;                      // second vector buffer (behind the factors)
      te_factor<KS>(dv, ev, m, th[b0 + lane], scal[3], lu + lane);
      for (int j = 0; j < m; ++j) {
        const uint32_t h = ((uint32_t)j * 2654435761u + (uint32_t)(b0 + lane) * 40503u + 12345u) >> 8;
        za[j * KS] = (float)(h & 0xffffu) * (1.f / 65536.f) - 0.5f;
      }
      // Three solves.  Between them the iterate is only rescaled by its largest magnitude (folded into the next solve's
      // first pass: the squares of the last normalisation cannot overflow, and nothing else depends on the length).
      float big = 1.f;
      for (int it = 0; it < 3; ++it) {
        te_forward<KS>(lu + lane, m, za, zb, (big > 0.f && big < INFINITY) ? 1.f / big : 1.f);
        big = te_backward<KS>(lu + lane, m, zb, za);
      }
      scal[8 + lane] = big;                                    // the waves of the back-transformation bring it to unit length
    }
    __syncthreads();
    float w0 = 0.f, w1 = 0.f;
    if (wave < kb) {
      w0 = (lane < m) ? zz[lane * KS + wave] : 0.f;
      w1 = (lane + 64 < m) ? zz[(lane + 64) * KS + wave] : 0.f;
      {
        // unit length (scaled by the largest magnitude first, so that the squares cannot overflow); this also clears what
        // is left of the start vector in blocks that S decouples from this eigenvalue (an exactly zero sub-diagonal
        // entry): some twenty orders of magnitude down, exact zeros in exact arithmetic
        const float big = scal[8 + wave];
        const float sc = (big > 0.f && big < INFINITY) ? 1.f / big : 1.f;
        w0 *= sc; w1 *= sc;
        const float nn = te_wave_sum(fmaf(w0, w0, w1 * w1));
        const float rn = (nn > 0.f) ? rsqrtf(nn) : 0.f;
        w0 *= rn; w1 *= rn;
        if (fabsf(w0) < 1e-12f) w0 = 0.f;
        if (fabsf(w1) < 1e-12f) w1 = 0.f;
      }
      // reflector j - 1 is fetched while reflector j is applied (the chain through w is all that is sequential)
      const float* r0p = Rf + min(lane, m - 1) * lt;
      const float* r1p = Rf + min(lane + 64, m - 1) * lt;
      float nb = (m >= 3) ? bet[m - 3] : 0.f, n0 = (m >= 3) ? r0p[m - 3] : 0.f, n1 = (m >= 3) ? r1p[m - 3] : 0.f;
      for (int j = m - 3; j >= 0; --j) {
        const float beta = nb;
        const float v0 = (lane > j && lane < m) ? n0 : 0.f;
        const float v1 = (lane + 64 > j && lane + 64 < m) ? n1 : 0.f;
        if (j > 0) { nb = bet[j - 1]; n0 = r0p[j - 1]; n1 = r1p[j - 1]; }
        const float s = beta * te_wave_sum(fmaf(v0, w0, v1 * w1));   // beta = 0: an identity reflector
        w0 = fmaf(-s, v0, w0); w1 = fmaf(-s, v1, w1);
      }
    }
    __syncthreads();                                           // every wave has read its column of zz / lu is free
    if (wave < kb) {
      if (lane < m) Wv[(b0 + wave) * m + lane] = w0;
      if (lane + 64 < m) Wv[(b0 + wave) * m + lane + 64] = w1;
    }
    __syncthreads();
  }
  if (wave == 0) {                                             // Gram-Schmidt over the k vectors, in order
    for (int i = 0; i < k; ++i) {
      float x0 = (lane < m) ? Wv[i * m + lane] : 0.f, x1 = (lane + 64 < m) ? Wv[i * m + lane + 64] : 0.f;
      for (int j = 0; j < i; ++j) {
        const float y0 = (lane < m) ? Wv[j * m + lane] : 0.f, y1 = (lane + 64 < m) ? Wv[j * m + lane + 64] : 0.f;
        const float dt = te_wave_sum(fmaf(x0, y0, x1 * y1));
        x0 = fmaf(-dt, y0, x0); x1 = fmaf(-dt, y1, x1);
      }
      const float nn = te_wave_sum(fmaf(x0, x0, x1 * x1));
      const float rn = (nn > 0.f) ? rsqrtf(nn) : 0.f;
      if (lane < m) Wv[i * m + lane] = x0 * rn;
      if (lane + 64 < m) Wv[i * m + lane + 64] = x1 * rn;
    }
  }
  __syncthreads();
  *theta = th;
  *W = Wv;
}

}  // namespace obf
