// Boundary refinement of TopK_B.  The fast score path works in fp32; two tokens whose exact
// attention masses (Eq. 1) differ by less than its error can come out in the wrong order at
// the selection threshold.  Here the few tokens whose float score lies within a relative band
// of the threshold are re-scored in double from the K / Qwin bits and the per-row
// log-sum-exp, and the retained slots inside the band are re-assigned by that exact order
// (ties to the lowest index).  Tokens outside the band keep their decision.
#include "boundary.hpp"

namespace obf {

constexpr int RF_THREADS = 256;
constexpr int RF_LAYER_THREADS = 1024;   // layerwise: one workgroup per layer re-scores the band in every head of the layer

template <int NW>
__device__ __forceinline__ int rf_block_exscan(int v, int& total, int* wsum) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
  for (int off = 1; off < 64; off <<= 1) {
    const int x = __shfl_up(inc, off);
    if (lane >= off) inc += x;
  }
  if (lane == 63) wsum[wave] = inc;
  __syncthreads();
  int pre = 0; total = 0;
  for (int wv = 0; wv < NW; ++wv) { if (wv < wave) pre += wsum[wv]; total += wsum[wv]; }
  __syncthreads();
  return pre + inc - v;
}

template <typename T, int NT>
__global__ __launch_bounds__(NT) void k_refine(const T* __restrict__ K, const T* __restrict__ Q,
                                                       const float* __restrict__ scores,
                                                       const double* __restrict__ row_lse, int N, int d, int R,
                                                       int max_budget, int32_t* __restrict__ idx,
                                                       const int32_t* __restrict__ n_keep,
                                                       int hps /*heads that share one selection: 1 (headwise) or the layer's heads; scores, idx, n_keep are per selection, K, Q, row_lse per head*/) {
  __shared__ uint32_t bitmap[kMaxTokens / 32];
  __shared__ int band[kBandCap];
  __shared__ double band_score[kBandCap];
  __shared__ int keep_new[kBandCap];
  __shared__ int wsum[(NT / 64)];
  __shared__ float wred[(NT / 64)];
  __shared__ int s_changed;
  const int head = blockIdx.x;
  const int n = n_keep[head];
  if (n <= 0 || n >= N) return;
  const float* sc = scores + (size_t)head * N;
  int32_t* out = idx + (size_t)head * max_budget;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

  // 1. threshold = smallest retained score
  float tmin = INFINITY;
  for (int i0 = threadIdx.x; i0 < n; i0 += 8 * NT) {      // batches of 8 independent index -> score loads
    int j[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) { const int i = i0 + q * NT; j[q] = (i < n) ? out[i] : -1; }
#pragma unroll
    for (int q = 0; q < 8; ++q) if (j[q] >= 0 && j[q] < N) tmin = fminf(tmin, sc[j[q]]);
  }
  for (int off = 32; off > 0; off >>= 1) tmin = fminf(tmin, __shfl_xor(tmin, off));
  if (lane == 0) wred[wave] = tmin;
  if (threadIdx.x == 0) s_changed = 0;
  __syncthreads();
  float tau = wred[0];
  for (int wv = 1; wv < (NT / 64); ++wv) tau = fminf(tau, wred[wv]);
  const float half = kBandRel * fabsf(tau);
  const float lo = tau - half, hi = tau + half;

  // 2. band tokens in index order (thread t owns a contiguous run of tokens; 16-byte loads when aligned)
  int seg = (N + NT - 1) / NT;
  seg = (seg + 3) & ~3;
  const int b0 = min(N, (int)threadIdx.x * seg), b1 = min(N, b0 + seg);
  const bool vec = (N & 3) == 0;
  int cnt = 0;
  if (vec) {
#pragma unroll 8
    for (int i = b0; i < b1; i += 4) {
      const float4 v = *(const float4*)(sc + i);
      cnt += (v.x >= lo && v.x <= hi) + (v.y >= lo && v.y <= hi) + (v.z >= lo && v.z <= hi) + (v.w >= lo && v.w <= hi);
    }
  } else {
    for (int i = b0; i < b1; ++i) { const float s = sc[i]; cnt += (s >= lo && s <= hi); }
  }
  int nband;
  int pos = rf_block_exscan<NT / 64>(cnt, nband, wsum);
  if (nband <= 1 || nband > kBandCap) return;
  if (cnt > 0) {
    for (int i = b0; i < b1; ++i) { const float s = sc[i]; if (s >= lo && s <= hi) band[pos++] = i; }
  }

  // 3. membership bitmap of the current retained set
  const int words = (N + 31) / 32;
  for (int i = threadIdx.x; i < words; i += NT) bitmap[i] = 0u;
  __syncthreads();
  for (int i = threadIdx.x; i < n; i += NT) { const int j = out[i]; atomicOr(&bitmap[j >> 5], 1u << (j & 31)); }
  __syncthreads();
  int kb = 0;
  if (threadIdx.x < nband) { const int j = band[threadIdx.x]; kb = (bitmap[j >> 5] >> (j & 31)) & 1u; }
  int nkb;
  rf_block_exscan<NT / 64>(kb, nkb, wsum);
  if (nkb == 0 || nkb == nband) return;

  // 4. exact scores of the band tokens
  rescore_band<T, (NT / 64)>(K + (size_t)head * hps * N * d, Q + (size_t)head * hps * R * d,
                            row_lse + (size_t)head * hps * R, d, R, band, nband, band_score);
  for (int h = 1; h < hps; ++h) {                      // layerwise: exact masses of the other heads, added in head order
    const size_t hh = (size_t)head * hps + h;
    rescore_band<T, (NT / 64), true>(K + hh * N * d, Q + hh * R * d, row_lse + hh * R, d, R, band, nband, band_score);
  }
  __syncthreads();

  // 5. the nkb best band tokens are retained
  if (threadIdx.x < nband) {
    const int keep = band_keeps(band_score, nband, nkb, threadIdx.x);
    keep_new[threadIdx.x] = keep;
    if (keep != kb) s_changed = 1;
  }
  __syncthreads();
  if (!s_changed) return;
  if (threadIdx.x < nband) {
    const int j = band[threadIdx.x];
    if (keep_new[threadIdx.x]) atomicOr(&bitmap[j >> 5], 1u << (j & 31));
    else atomicAnd(&bitmap[j >> 5], ~(1u << (j & 31)));
  }
  __syncthreads();

  // 6. rewrite the ascending index list from the bitmap
  const int wseg = (words + NT - 1) / NT;
  const int w0 = min(words, (int)threadIdx.x * wseg), w1 = min(words, w0 + wseg);
  int pc = 0;
  for (int wi = w0; wi < w1; ++wi) pc += __popc(bitmap[wi]);
  int total;
  int o = rf_block_exscan<NT / 64>(pc, total, wsum);
  for (int wi = w0; wi < w1; ++wi) {
    uint32_t bits = bitmap[wi];
    while (bits) {
      const int bpos = __ffs(bits) - 1;
      bits &= bits - 1;
      out[o++] = wi * 32 + bpos;
    }
  }
}

obf_status_t launch_refine(const Dims& m, const Workspace& w, char* ws, const void* K, const void* Q,
                           const float* scores, const double* row_lse, int32_t max_budget, int32_t* idx,
                           const int32_t* n_keep, hipStream_t st) {
  (void)w; (void)ws;
  if (m.dtype == OBF_BF16)
    { ProfScope prof_(ST_REFINE, st); hipLaunchKernelGGL((k_refine<uint16_t, RF_THREADS>), dim3(m.heads), dim3(RF_THREADS), 0, st, (const uint16_t*)K, (const uint16_t*)Q,
                       scores, row_lse, m.N, m.d, m.R, max_budget, idx, n_keep, 1); }
  else
    { ProfScope prof_(ST_REFINE, st); hipLaunchKernelGGL((k_refine<float, RF_THREADS>), dim3(m.heads), dim3(RF_THREADS), 0, st, (const float*)K, (const float*)Q, scores,
                       row_lse, m.N, m.d, m.R, max_budget, idx, n_keep, 1); }
  return check_launch("refine");
}

// The same re-decision for selections shared by the heads of a layer: scores, idx and n_keep are per layer.
obf_status_t launch_refine_layers(const Dims& m, const void* K, const void* Q, const float* layer_scores,
                                  const double* row_lse, int32_t max_budget, int32_t* idx_layer,
                                  const int32_t* n_keep_layer, hipStream_t st) {
  ProfScope prof_(ST_REFINE, st);
  if (m.dtype == OBF_BF16)
    hipLaunchKernelGGL((k_refine<uint16_t, RF_LAYER_THREADS>), dim3(m.L), dim3(RF_LAYER_THREADS), 0, st, (const uint16_t*)K, (const uint16_t*)Q,
                       layer_scores, row_lse, m.N, m.d, m.R, max_budget, idx_layer, n_keep_layer, m.H);
  else
    hipLaunchKernelGGL((k_refine<float, RF_LAYER_THREADS>), dim3(m.L), dim3(RF_LAYER_THREADS), 0, st, (const float*)K, (const float*)Q,
                       layer_scores, row_lse, m.N, m.d, m.R, max_budget, idx_layer, n_keep_layer, m.H);
  return check_launch("refine (layerwise)");
}

}  // namespace obf
