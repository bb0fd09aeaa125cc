// Gather of the retained rows (Alg. 2 line 7): K_out = K[idx], V_out = V[idx], bit copies in
// 16-byte pieces; rows past n_keep are zero-filled so the padded output is deterministic.
#include "common.hpp"

namespace obf {

constexpr int GA_THREADS = 256;

__global__ __launch_bounds__(GA_THREADS) void k_gather(const uint4* __restrict__ K, const uint4* __restrict__ V,
                                                       const int32_t* __restrict__ idx,
                                                       const int32_t* __restrict__ n_keep, int N, int row_vec /*uint4 per row*/,
                                                       int max_budget, uint4* __restrict__ K_out, uint4* __restrict__ V_out) {
  const int head = blockIdx.y;
  const int rows_per_block = GA_THREADS / row_vec;
  const int r = blockIdx.x * rows_per_block + threadIdx.x / row_vec;
  const int c = threadIdx.x % row_vec;
  if (r >= max_budget) return;
  const int n = n_keep[head];
  const size_t o = ((size_t)head * max_budget + r) * row_vec + c;
  uint4 kv = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
  if (r < n) {
    const int j = idx[(size_t)head * max_budget + r];
    const size_t s = ((size_t)head * N + j) * row_vec + c;
    if (K_out) kv = K[s];
    if (V_out) vv = V[s];
  }
  if (K_out) K_out[o] = kv;
  if (V_out) V_out[o] = vv;
}

obf_status_t launch_gather(const Dims& m, const void* K, const void* V, const int32_t* idx, const int32_t* n_keep,
                           int32_t max_budget, void* K_out, void* V_out, hipStream_t st) {
  if (max_budget == 0 || (!K_out && !V_out)) return OBF_OK;
  const int row_vec = m.d * m.esize / 16;            // 8, 16 or 32
  const int rows_per_block = GA_THREADS / row_vec;
  dim3 grid((max_budget + rows_per_block - 1) / rows_per_block, m.heads);
  { ProfScope prof_(ST_GATHER, st); hipLaunchKernelGGL(k_gather, grid, dim3(GA_THREADS), 0, st, (const uint4*)K, (const uint4*)V, idx, n_keep, m.N, row_vec,
                     max_budget, (uint4*)K_out, (uint4*)V_out); }
  return check_launch("gather");
}

}  // namespace obf
