// TopK_B (Sec. 4.3.2): the B largest scores of a head, ties to the lowest index, written as an
// ascending index list.  One workgroup per head; the N keys live in LDS.  All comparisons are
// on an order-preserving integer image of the fp32 bit patterns, so the result is exact.
#include "common.hpp"

namespace obf {

constexpr int SEL_THREADS = 1024;
constexpr int SEL_WAVES = SEL_THREADS / 64;
constexpr int SEL_BATCH = 256;   // heads per launch when budgets differ per head

struct BudgetBatch { int32_t b[SEL_BATCH]; };

// larger float <=> larger key (total order on the bit patterns; -0 < +0)
__device__ __forceinline__ uint32_t order_key(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// exclusive prefix sums of (a, b) over the workgroup, in thread order
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

__global__ __launch_bounds__(SEL_THREADS) void k_select(const float* __restrict__ scores, int N, int head0,
                                                        int uniform_budget, BudgetBatch per_head, int use_per_head,
                                                        int max_budget, int32_t* __restrict__ idx,
                                                        int32_t* __restrict__ n_keep) {
  extern __shared__ uint32_t keys[];           // [N]
  __shared__ int hist[256];
  __shared__ int wsum[2 * SEL_WAVES];
  __shared__ uint32_t s_prefix;
  __shared__ int s_remaining;
  const int head = head0 + blockIdx.x;
  const float* sc = scores + (size_t)head * N;
  int32_t* out = idx + (size_t)head * max_budget;
  int B = use_per_head ? per_head.b[blockIdx.x] : uniform_budget;
  if (B > N) B = N;

  if (B == 0 || B == N) {
    for (int i = threadIdx.x; i < max_budget; i += SEL_THREADS) out[i] = (i < B) ? i : -1;
    if (threadIdx.x == 0) n_keep[head] = B;
    return;
  }
  for (int i = threadIdx.x; i < N; i += SEL_THREADS) keys[i] = order_key(sc[i]);
  if (threadIdx.x == 0) { s_prefix = 0u; s_remaining = B; }
  __syncthreads();

  // radix select, most significant byte first: find the key T of rank B (1-based, descending)
  uint32_t mask = 0u;
  for (int shift = 24; shift >= 0; shift -= 8) {
    for (int i = threadIdx.x; i < 256; i += SEL_THREADS) hist[i] = 0;
    __syncthreads();
    const uint32_t prefix = s_prefix;
    for (int i = threadIdx.x; i < N; i += SEL_THREADS) {
      const uint32_t k = keys[i];
      if ((k & mask) == prefix) atomicAdd(&hist[(k >> shift) & 255u], 1);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      int rem = s_remaining, bin = 255;
      for (; bin > 0; --bin) {
        const int c = hist[bin];
        if (c >= rem) break;
        rem -= c;
      }
      s_remaining = rem;
      s_prefix = prefix | ((uint32_t)bin << shift);
    }
    mask |= 255u << shift;
    __syncthreads();
  }
  const uint32_t T = s_prefix;
  const int need_eq = s_remaining;     // how many keys equal to T are kept (the lowest indices)

  // ordered compaction: thread t owns tokens [t*seg, (t+1)*seg)
  const int seg = (N + SEL_THREADS - 1) / SEL_THREADS;
  const int b0 = min(N, (int)threadIdx.x * seg), b1 = min(N, b0 + seg);
  int cg = 0, ce = 0;
  for (int i = b0; i < b1; ++i) { const uint32_t k = keys[i]; cg += (k > T); ce += (k == T); }
  int eg, ee, tg, te;
  block_exscan2(cg, ce, eg, ee, tg, te, wsum);
  for (int i = b0; i < b1; ++i) {
    const uint32_t k = keys[i];
    if (k > T) { out[eg + min(ee, need_eq)] = i; ++eg; }
    else if (k == T) { if (ee < need_eq) out[eg + ee] = i; ++ee; }
  }
  for (int i = B + threadIdx.x; i < max_budget; i += SEL_THREADS) out[i] = -1;
  if (threadIdx.x == 0) n_keep[head] = B;
}

obf_status_t launch_select(const Dims& m, const float* scores, const int32_t* budgets_host, int32_t budget,
                           int32_t max_budget, int32_t* idx, int32_t* n_keep, hipStream_t st) {
  const size_t smem = sizeof(uint32_t) * (size_t)m.N;
  static bool attr_done = false;
  if (!attr_done) {
    (void)hipFuncSetAttribute((const void*)k_select, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxTokens * 4);
    attr_done = true;
  }
  BudgetBatch bb;
  if (!budgets_host) {
    { ProfScope prof_(ST_SELECT, st); hipLaunchKernelGGL(k_select, dim3(m.heads), dim3(SEL_THREADS), smem, st, scores, m.N, 0, budget, bb, 0, max_budget,
                       idx, n_keep); }
    return check_launch("select");
  }
  for (int h0 = 0; h0 < m.heads; h0 += SEL_BATCH) {
    const int nb = (m.heads - h0 < SEL_BATCH) ? (m.heads - h0) : SEL_BATCH;
    for (int i = 0; i < nb; ++i) bb.b[i] = budgets_host[h0 + i];
    { ProfScope prof_(ST_SELECT, st); hipLaunchKernelGGL(k_select, dim3(nb), dim3(SEL_THREADS), smem, st, scores, m.N, h0, 0, bb, 1, max_budget, idx, n_keep); }
    if (check_launch("select") != OBF_OK) return OBF_ERR_HIP;
  }
  return OBF_OK;
}

}  // namespace obf
