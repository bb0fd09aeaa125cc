// TopK_B (Sec. 4.3.2): the B largest scores of a head, ties to the lowest index, written as an
// ascending index list.  One workgroup per head; the N keys live in registers.  All comparisons are
// on an order-preserving integer image of the fp32 bit patterns, so the result is exact.
#include "boundary.hpp"

namespace obf {

constexpr int SEL_BATCH = 896;   // heads per launch when budgets differ per head (the budgets travel as a kernel argument: 3.5 KB of the 4 KB)

struct BudgetBatch { int32_t b[SEL_BATCH]; };

// larger float <=> larger key (total order on the bit patterns; -0 < +0)
__device__ __forceinline__ uint32_t order_key(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float key_to_float(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// exclusive prefix sums of (a, b) over the workgroup, in thread order
template <int SEL_WAVES>
__device__ __forceinline__ void block_exscan2(int a, int b, int& ea, int& eb, int& ta, int& tb, int* wsum /*[2*SEL_WAVES]*/) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int ia = a, ib = b;
  for (int off = 1; off < 64; off <<= 1) {
    const int xa = __shfl_up(ia, off), xb = __shfl_up(ib, off);
    if (lane >= off) { ia += xa; ib += xb; }
  }
  if (lane == 63) { wsum[wave] = ia; wsum[SEL_WAVES + wave] = ib; }
  __syncthreads();
  int pa = 0, pb = 0;
  ta = 0; tb = 0;
  for (int wv = 0; wv < SEL_WAVES; ++wv) {
    const int sa = wsum[wv], sb = wsum[SEL_WAVES + wv];
    if (wv < wave) { pa += sa; pb += sb; }
    ta += sa; tb += sb;
  }
  ea = pa + ia - a; eb = pb + ib - b;
  __syncthreads();
}

// Thread t owns the SEG consecutive tokens starting at t*SEG (keys stay in registers).  The key of rank B is
// found by bisection on the 32 key bits, most significant first: T is the largest value with
// count(key >= T) >= B.  Counting is one ballot + population count per owned token and one workgroup sum per bit.
// With REFINE the tokens whose score lies in the relative band around the threshold are re-decided in double from K, Q
// and the row log-sum-exp before the list is written (same decisions as select followed by the refinement kernel).
template <int SEG, int SEL_THREADS, bool REFINE, typename ET>
__global__ __launch_bounds__(SEL_THREADS) void k_select(const float* __restrict__ scores, int N, int head0,
                                                        int uniform_budget, BudgetBatch per_head, int use_per_head,
                                                        int max_budget, int32_t* __restrict__ idx,
                                                        int32_t* __restrict__ n_keep, const ET* __restrict__ K,
                                                        const ET* __restrict__ Q, const double* __restrict__ row_lse,
                                                        int d, int R, int scs, int kvs,
                                                        int32_t* __restrict__ sel_flags /*nullable; written with REFINE only*/) {
  constexpr int SEL_WAVES = SEL_THREADS / 64;
  __shared__ int band[REFINE ? kBandCap : 1];
  __shared__ double band_score[REFINE ? kBandCap : 1];
  __shared__ int keep_new[REFINE ? kBandCap : 1];
  __shared__ int s_changed;
  __shared__ int wcnt[2][SEL_WAVES];
  __shared__ int wsum[2 * SEL_WAVES];
  const int head = head0 + blockIdx.x;
  const float* sc = scores + (size_t)head * scs;
  int32_t* out = idx + (size_t)head * max_budget;
  int B = use_per_head ? per_head.b[blockIdx.x] : uniform_budget;
  if (B > N) B = N;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  if (B == 0 || B == N) {
    for (int i = tid; i < max_budget; i += SEL_THREADS) out[i] = (i < B) ? i : -1;
    if (tid == 0) n_keep[head] = B;
    return;
  }
  const int base = tid * SEG;
  uint32_t key[SEG];
  int nvalid = min(SEG, max(0, N - base));                     // tokens of this thread inside the head
  if (nvalid == SEG && (((uintptr_t)(sc + base) & 15) == 0)) {
#pragma unroll
    for (int i = 0; i < SEG; i += 4) {
      const float4 v = *(const float4*)(sc + base + i);
      key[i] = order_key(v.x); key[i + 1] = order_key(v.y); key[i + 2] = order_key(v.z); key[i + 3] = order_key(v.w);
    }
  } else {
#pragma unroll
    for (int i = 0; i < SEG; ++i) key[i] = (i < nvalid) ? order_key(sc[base + i]) : 0u;
  }

  // tokens outside the head carry key 0 and every candidate is >= 1, so they never count
  auto count_ge = [&](uint32_t cand, int buf) -> int {
    int c = 0;
#pragma unroll
    for (int i = 0; i < SEG; ++i) c += __popcll(__ballot(key[i] >= cand));
    if (lane == 0) wcnt[buf][wave] = c;
    __syncthreads();
    int tot = 0;
#pragma unroll
    for (int w = 0; w < SEL_WAVES; ++w) tot += wcnt[buf][w];
    return tot;
  };

  // Bisection, most significant bit first.  As soon as exactly B keys are >= the candidate, the retained set is
  // known and the rank-B key is the smallest of them (one more workgroup reduction) - the remaining bits are skipped.
  uint32_t T = 0u;
  int buf = 0;
  bool exact = false;
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t cand = T | (1u << bit);
    const int c = count_ge(cand, buf);
    buf ^= 1;
    if (c >= B) T = cand;
    if (c == B) { exact = true; break; }
  }
  if (exact) {
    uint32_t mn = 0xffffffffu;
#pragma unroll
    for (int i = 0; i < SEG; ++i) if (i < nvalid && key[i] >= T) mn = min(mn, key[i]);
    for (int off = 32; off > 0; off >>= 1) mn = min(mn, (uint32_t)__shfl_xor((int)mn, off));
    if (lane == 0) wcnt[buf][wave] = (int)mn;
    __syncthreads();
    uint32_t t = 0xffffffffu;
#pragma unroll
    for (int w = 0; w < SEL_WAVES; ++w) t = min(t, (uint32_t)wcnt[buf][w]);
    T = t;
    buf ^= 1;
  }
  // keys greater than T are all kept; of the keys equal to T the lowest indices fill the rest
  int n_gt = 0;
  if (T != 0xffffffffu) n_gt = count_ge(T + 1u, buf);
  buf ^= 1;
  const int need_eq = B - n_gt;
  int cg = 0, ce = 0;
#pragma unroll
  for (int i = 0; i < SEG; ++i) { if (i < nvalid) { cg += (key[i] > T); ce += (key[i] == T); } }
  int eg, ee, tg, te;
  block_exscan2<SEL_WAVES>(cg, ce, eg, ee, tg, te, wsum);
  bool refined = false;
  int bpos0 = 0;
  float lo = 0.f, hi = 0.f;
  if (REFINE) {
    // band around the threshold score, in the same float arithmetic as the standalone refinement
    const float tau = key_to_float(T);
    const float half = kBandRel * fabsf(tau);
    lo = tau - half; hi = tau + half;
    int cb = 0, ckb = 0;
    {
      int er = ee;                                      // running count of keys equal to T before this token
#pragma unroll
      for (int i = 0; i < SEG; ++i) {
        if (i < nvalid) {
          const uint32_t k = key[i];
          const float s = key_to_float(k);
          const bool kept = (k > T) || (k == T && er < need_eq);
          er += (k == T);
          if (s >= lo && s <= hi) { ++cb; ckb += kept; }
        }
      }
    }
    int ebk, nband, nkb;
    block_exscan2<SEL_WAVES>(cb, ckb, bpos0, ebk, nband, nkb, wsum);
    if (tid == 0) s_changed = 0;
    // a band that straddles the threshold but is too large to re-score keeps the single-precision order: say so
    if (sel_flags && tid == 0) sel_flags[head] = (nband > kBandCap && nkb > 0 && nkb < nband) ? OBF_SELECT_BAND_OVERFLOW : 0;
    if (nband > 1 && nband <= kBandCap && nkb > 0 && nkb < nband) {       // uniform
      int bp = bpos0, er = ee;
#pragma unroll
      for (int i = 0; i < SEG; ++i) {
        if (i < nvalid) {
          const uint32_t k = key[i];
          const float s = key_to_float(k);
          const bool kept = (k > T) || (k == T && er < need_eq);
          er += (k == T);
          if (s >= lo && s <= hi) { band[bp] = base + i; keep_new[bp] = kept; ++bp; }
        }
      }
      __syncthreads();
      rescore_band<ET, SEL_WAVES>(K + (size_t)head * kvs * d, Q + (size_t)head * R * d, row_lse + (size_t)head * R, d, R,
                                 band, nband, band_score);
      __syncthreads();
      int keep = 0, was = 0;
      if (tid < nband) { was = keep_new[tid]; keep = band_keeps(band_score, nband, nkb, tid); if (keep != was) s_changed = 1; }
      __syncthreads();
      if (tid < nband) keep_new[tid] = keep;
      __syncthreads();
      refined = s_changed != 0;
    }
  }
  if (!refined) {
#pragma unroll
    for (int i = 0; i < SEG; ++i) {
      if (i < nvalid) {
        const uint32_t k = key[i];
        if (k > T) { out[eg + min(ee, need_eq)] = base + i; ++eg; }
        else if (k == T) { if (ee < need_eq) out[eg + ee] = base + i; ++ee; }
      }
    }
  } else {
    // membership changed inside the band: recount positions from the final flags
    uint32_t flags = 0u;
    int cnt = 0;
    {
      int bp = bpos0, er = ee;
#pragma unroll
      for (int i = 0; i < SEG; ++i) {
        if (i < nvalid) {
          const uint32_t k = key[i];
          const float s = key_to_float(k);
          bool kept = (k > T) || (k == T && er < need_eq);
          er += (k == T);
          if (s >= lo && s <= hi) { kept = keep_new[bp] != 0; ++bp; }
          if (kept) { flags |= 1u << i; ++cnt; }
        }
      }
    }
    int e0, e1, t0, t1;
    block_exscan2<SEL_WAVES>(cnt, 0, e0, e1, t0, t1, wsum);
#pragma unroll
    for (int i = 0; i < SEG; ++i) if (flags & (1u << i)) out[e0++] = base + i;
  }
  for (int i = B + tid; i < max_budget; i += SEL_THREADS) out[i] = -1;
  if (tid == 0) n_keep[head] = B;
}

template <int SEG, int SEL_THREADS, bool REFINE, typename T>
static obf_status_t launch_select_seg(const Dims& m, const float* scores, const int32_t* budgets_host, int32_t budget,
                                      int32_t max_budget, int32_t* idx, int32_t* n_keep, const void* K, const void* Q,
                                      const double* row_lse, hipStream_t st, int32_t* sel_flags) {
  BudgetBatch bb;
  if (!budgets_host) {
    { ProfScope prof_(ST_SELECT, st);
      hipLaunchKernelGGL((k_select<SEG, SEL_THREADS, REFINE, T>), dim3(m.heads), dim3(SEL_THREADS), 0, st, scores, m.N, 0,
                         budget, bb, 0, max_budget, idx, n_keep, (const T*)K, (const T*)Q, row_lse, m.d, m.R, m.scs, m.kvs, sel_flags); }
    return check_launch("select");
  }
  for (int h0 = 0; h0 < m.heads; h0 += SEL_BATCH) {
    const int nb = (m.heads - h0 < SEL_BATCH) ? (m.heads - h0) : SEL_BATCH;
    for (int i = 0; i < nb; ++i) bb.b[i] = budgets_host[h0 + i];
    { ProfScope prof_(ST_SELECT, st);
      hipLaunchKernelGGL((k_select<SEG, SEL_THREADS, REFINE, T>), dim3(nb), dim3(SEL_THREADS), 0, st, scores, m.N, h0, 0, bb,
                         1, max_budget, idx, n_keep, (const T*)K, (const T*)Q, row_lse, m.d, m.R, m.scs, m.kvs, sel_flags); }
    if (check_launch("select") != OBF_OK) return OBF_ERR_HIP;
  }
  return OBF_OK;
}

template <bool REFINE, typename T>
static obf_status_t dispatch_select(const Dims& m, const float* scores, const int32_t* budgets_host, int32_t budget,
                                    int32_t max_budget, int32_t* idx, int32_t* n_keep, const void* K, const void* Q,
                                    const double* row_lse, hipStream_t st, int32_t* sel_flags) {
  // per bit every wave counts its keys and the workgroup adds the counts: 16 keys per thread up to 8192 tokens, 32 above
#define OBF_SEL(SEG, THR) launch_select_seg<SEG, THR, REFINE, T>(m, scores, budgets_host, budget, max_budget, idx, n_keep, K, Q, row_lse, st, sel_flags)
  if (m.N <= 4 * 256) return OBF_SEL(4, 256);
  if (m.N <= 8 * 256) return OBF_SEL(8, 256);
  if (m.N <= 16 * 256) return OBF_SEL(16, 256);
  if (m.N <= 16 * 512) return OBF_SEL(16, 512);      // 8192 tokens: 37 us against 42 with (32, 256) and 48 with (8, 1024)
  if (m.N <= 32 * 512) return OBF_SEL(32, 512);
  return OBF_SEL(32, 1024);
#undef OBF_SEL
}

obf_status_t launch_select(const Dims& m, const float* scores, const int32_t* budgets_host, int32_t budget,
                           int32_t max_budget, int32_t* idx, int32_t* n_keep, hipStream_t st) {
  return dispatch_select<false, float>(m, scores, budgets_host, budget, max_budget, idx, n_keep, nullptr, nullptr, nullptr, st, nullptr);
}

obf_status_t launch_select_refine(const Dims& m, const float* scores, const int32_t* budgets_host, int32_t budget,
                                  int32_t max_budget, int32_t* idx, int32_t* n_keep, const void* K, const void* Q,
                                  const double* row_lse, hipStream_t st, int32_t* sel_flags) {
  if (m.dtype == OBF_BF16)
    return dispatch_select<true, uint16_t>(m, scores, budgets_host, budget, max_budget, idx, n_keep, K, Q, row_lse, st, sel_flags);
  return dispatch_select<true, float>(m, scores, budgets_host, budget, max_budget, idx, n_keep, K, Q, row_lse, st, sel_flags);
}

__global__ void k_diag_flags(obf_diag_t* __restrict__ diag, const int32_t* __restrict__ sel_flags, int heads) {
  const int h = blockIdx.x * blockDim.x + threadIdx.x;
  if (h < heads) diag[h].select_flags = sel_flags[h];
}

obf_status_t launch_diag_flags(obf_diag_t* diag, const int32_t* sel_flags, int heads, hipStream_t st) {
  if (!diag || !sel_flags || heads <= 0) return OBF_OK;
  hipLaunchKernelGGL(k_diag_flags, dim3((heads + 255) / 256), dim3(256), 0, st, diag, sel_flags, heads);
  return check_launch("diag flags");
}

}  // namespace obf
