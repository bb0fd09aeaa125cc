// Layerwise granularity of the retention rule (Sec. 4.3.2): one index set per layer, TopK_B of the attention mass
// summed over the layer's heads, shared by all of them.  The per-head scores, the gather and Orthogonal BackFill
// are the headwise ones; only the selection differs.
#include "common.hpp"

namespace obf {

constexpr int LW_THREADS = 256;

// layer_scores[l][j] = sum over the heads h of the layer (in head order) of scores[l][h][j]
__global__ __launch_bounds__(LW_THREADS) void k_layer_sum(const float* __restrict__ scores, float* __restrict__ out,
                                                          int H, int N, int scs) {
  const int l = blockIdx.y;
  const int j = blockIdx.x * LW_THREADS + threadIdx.x;
  if (j >= N) return;
  const float* p = scores + (size_t)l * H * scs + j;
  float s = 0.f;
  for (int h = 0; h < H; ++h) s += p[(size_t)h * scs];
  out[(size_t)l * N + j] = s;
}

// idx[l][h][:] = idx_layer[l][:], n_keep[l][h] = n_keep_layer[l]
__global__ __launch_bounds__(LW_THREADS) void k_share_selection(const int32_t* __restrict__ idx_layer,
                                                                const int32_t* __restrict__ n_keep_layer, int H,
                                                                int max_budget, int32_t* __restrict__ idx,
                                                                int32_t* __restrict__ n_keep) {
  const int head = blockIdx.y, l = head / H;
  const int i = blockIdx.x * LW_THREADS + threadIdx.x;
  if (i < max_budget) idx[(size_t)head * max_budget + i] = idx_layer[(size_t)l * max_budget + i];
  if (i == 0) n_keep[head] = n_keep_layer[l];
}

obf_status_t launch_select_layerwise(const Dims& m, const Workspace& w, char* ws, const float* scores,
                                     const int32_t* budgets_host, int32_t budget, int32_t max_budget, int32_t* idx,
                                     int32_t* n_keep, const void* K, const void* Q, const double* row_lse,
                                     hipStream_t st) {
  float* layer_scores = (float*)(ws + w.layer_scores);
  int32_t* idx_layer = (int32_t*)(ws + w.layer_idx);
  int32_t* nk_layer = idx_layer + (size_t)m.L * (max_budget > 0 ? max_budget : 0);
  {
    ProfScope prof_(ST_SELECT, st);
    hipLaunchKernelGGL(k_layer_sum, dim3((m.N + LW_THREADS - 1) / LW_THREADS, m.L), dim3(LW_THREADS), 0, st, scores,
                       layer_scores, m.H, m.N, m.scs);
  }
  if (check_launch("layer sum") != OBF_OK) return OBF_ERR_HIP;
  Dims ml = m;
  ml.heads = m.L;                                       // one selection per layer
  ml.scs = m.N;                                         // the layer sums are dense
  if (launch_select(ml, layer_scores, budgets_host, budget, max_budget, idx_layer, nk_layer, st) != OBF_OK) return OBF_ERR_HIP;
  double* part = (double*)(ws + w.band);               // [heads][kBandCap] exact masses of the band tokens, per head
  if (launch_refine_layers(m, K, Q, layer_scores, row_lse, max_budget, idx_layer, nk_layer, part, st) != OBF_OK) return OBF_ERR_HIP;
  {
    ProfScope prof_(ST_SELECT, st);
    hipLaunchKernelGGL(k_share_selection, dim3((max(max_budget, 1) + LW_THREADS - 1) / LW_THREADS, m.heads), dim3(LW_THREADS),
                       0, st, idx_layer, nk_layer, m.H, max_budget, idx, n_keep);
  }
  return check_launch("share selection");
}

}  // namespace obf
