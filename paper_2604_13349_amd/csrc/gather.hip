// Gather of the retained rows (the gather step of Alg. 2): K_out = K[idx], V_out = V[idx], bit copies in
// 16-byte pieces; rows past n_keep are zero-filled so the padded output is deterministic.
#include "common.hpp"

namespace obf {

constexpr int GA_THREADS = 256;
constexpr int GA_UNROLL = 4;             // rows per thread

__global__ __launch_bounds__(GA_THREADS) void k_gather(const uint4* __restrict__ K, const uint4* __restrict__ V,
                                                       const int32_t* __restrict__ idx,
                                                       const int32_t* __restrict__ n_keep, int kvs /*tokens per head in K, V*/, int row_vec /*uint4 per row*/,
                                                       int max_budget, uint4* __restrict__ K_out, uint4* __restrict__ V_out,
                                                       double* __restrict__ fro_part /*bf16 rows of 256 bytes only*/) {
  __shared__ float s_red[GA_THREADS / 64];
  const int head = blockIdx.y;
  const int rows_per_pass = GA_THREADS / row_vec;
  const int r0 = blockIdx.x * rows_per_pass * GA_UNROLL + threadIdx.x / row_vec;
  const int c = threadIdx.x % row_vec;
  const int n = n_keep[head];
  // GA_UNROLL rows per thread, all loads issued before the first store
  int j[GA_UNROLL];
#pragma unroll
  for (int u = 0; u < GA_UNROLL; ++u) {
    const int r = r0 + u * rows_per_pass;
    j[u] = (r < n && r < max_budget) ? idx[(size_t)head * max_budget + r] : -1;
  }
  uint4 kv[GA_UNROLL], vv[GA_UNROLL];
#pragma unroll
  for (int u = 0; u < GA_UNROLL; ++u) {
    kv[u] = make_uint4(0, 0, 0, 0); vv[u] = make_uint4(0, 0, 0, 0);
    if (j[u] >= 0) {
      const size_t s = ((size_t)head * kvs + j[u]) * row_vec + c;
      if (K_out) kv[u] = K[s];
      if (V_out) vv[u] = V[s];
    }
  }
#pragma unroll
  for (int u = 0; u < GA_UNROLL; ++u) {
    const int r = r0 + u * rows_per_pass;
    if (r < max_budget) {
      const size_t o = ((size_t)head * max_budget + r) * row_vec + c;
      if (K_out) K_out[o] = kv[u];
      if (V_out) V_out[o] = vv[u];
    }
  }
  if (fro_part) {
    // sum of squares of this workgroup's V rows (zero for the padding), in a fixed order
    float sq = 0.f;
#pragma unroll
    for (int u = 0; u < GA_UNROLL; ++u) {
      const uint32_t w4[4] = {vv[u].x, vv[u].y, vv[u].z, vv[u].w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float a = __uint_as_float(w4[i] << 16), b = __uint_as_float(w4[i] & 0xffff0000u);
        sq = fmaf(a, a, sq); sq = fmaf(b, b, sq);
      }
    }
    for (int off = 32; off > 0; off >>= 1) sq += __shfl_xor(sq, off);
    if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = sq;
    __syncthreads();
    if (threadIdx.x == 0)
      fro_part[(size_t)head * gridDim.x + blockIdx.x] = ((double)s_red[0] + (double)s_red[1]) + ((double)s_red[2] + (double)s_red[3]);
  }
}

obf_status_t launch_gather(const Dims& m, const void* K, const void* V, const int32_t* idx, const int32_t* n_keep,
                           int32_t max_budget, void* K_out, void* V_out, hipStream_t st, double* fro_part) {
  if (max_budget == 0 || (!K_out && !V_out)) return OBF_OK;
  if (!(m.dtype == OBF_BF16 && m.d * m.esize == 256 && V_out)) fro_part = nullptr;
  const int row_vec = m.d * m.esize / 16;            // 8, 16 or 32
  const int rows_per_block = GA_UNROLL * GA_THREADS / row_vec;
  dim3 grid((max_budget + rows_per_block - 1) / rows_per_block, m.heads);
  { ProfScope prof_(ST_GATHER, st); hipLaunchKernelGGL(k_gather, grid, dim3(GA_THREADS), 0, st, (const uint4*)K, (const uint4*)V, idx, n_keep, m.kvs, row_vec,
                     max_budget, (uint4*)K_out, (uint4*)V_out, fro_part); }
  return check_launch("gather");
}

// Index lists of a token window back in the head's own numbering: valid entries move by `offset`, the -1 padding stays.
__global__ __launch_bounds__(GA_THREADS) void k_idx_offset(int32_t* __restrict__ idx, size_t n, int32_t offset) {
  const size_t i = (size_t)blockIdx.x * GA_THREADS + threadIdx.x;
  if (i < n) { const int32_t v = idx[i]; if (v >= 0) idx[i] = v + offset; }
}

obf_status_t launch_idx_offset(int32_t* idx, size_t n, int32_t offset, hipStream_t st) {
  if (n == 0 || offset == 0) return OBF_OK;
  hipLaunchKernelGGL(k_idx_offset, dim3((unsigned)((n + GA_THREADS - 1) / GA_THREADS)), dim3(GA_THREADS), 0, st, idx, n, offset);
  return check_launch("idx offset");
}

}  // namespace obf
