// Boundary refinement of TopK_B.  The fast score path works in fp32; two tokens whose exact
// attention masses (Eq. 1) differ by less than its error can come out in the wrong order at
// the selection threshold.  Here the few tokens whose float score lies within a relative band
// of the threshold are re-scored in double from the K / Qwin bits and the per-row
// log-sum-exp, and the retained slots inside the band are re-assigned by that exact order
// (ties to the lowest index).  Tokens outside the band keep their decision.
#include "boundary.hpp"

namespace obf {

constexpr int RF_THREADS = 256;

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

template <int NT>
struct RfShared {
  uint32_t bitmap[kMaxTokens / 32];
  int band[kBandCap];
  double band_score[kBandCap];
  int keep_new[kBandCap];
  int wsum[NT / 64];
  float wred[NT / 64];
  int s_changed;
};

// Steps 1-3: the threshold (smallest retained score), the band tokens in index order, the membership bitmap of
// the current retained set.  Returns false when there is nothing to re-decide.  kb (threads < nband): is band
// token threadIdx.x retained now; nkb: how many band tokens are.
template <int NT>
__device__ bool rf_find_band(RfShared<NT>& sh, const float* __restrict__ sc, const int32_t* __restrict__ out, int n,
                             int N, int& nband, int& nkb, int& kb) {
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
  if (lane == 0) sh.wred[wave] = tmin;
  if (threadIdx.x == 0) sh.s_changed = 0;
  __syncthreads();
  float tau = sh.wred[0];
  for (int wv = 1; wv < NT / 64; ++wv) tau = fminf(tau, sh.wred[wv]);
  const float half = kBandRel * fabsf(tau);
  const float lo = tau - half, hi = tau + half;

  // 2. band tokens in index order (thread t owns a contiguous run of tokens; 16-byte loads when aligned)
  int seg = (N + NT - 1) / NT;
  seg = (seg + 3) & ~3;
  const int b0 = min(N, (int)threadIdx.x * seg), b1 = min(N, b0 + seg);
  const bool vec = (N & 3) == 0 && ((uintptr_t)sc & 15) == 0;
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
  int pos = rf_block_exscan<NT / 64>(cnt, nband, sh.wsum);
  if (nband <= 1 || nband > kBandCap) return false;
  if (cnt > 0) {
    for (int i = b0; i < b1; ++i) { const float s = sc[i]; if (s >= lo && s <= hi) sh.band[pos++] = i; }
  }

  // 3. membership bitmap of the current retained set
  const int words = (N + 31) / 32;
  for (int i = threadIdx.x; i < words; i += NT) sh.bitmap[i] = 0u;
  __syncthreads();
  for (int i = threadIdx.x; i < n; i += NT) { const int j = out[i]; atomicOr(&sh.bitmap[j >> 5], 1u << (j & 31)); }
  __syncthreads();
  kb = 0;
  if ((int)threadIdx.x < nband) { const int j = sh.band[threadIdx.x]; kb = (sh.bitmap[j >> 5] >> (j & 31)) & 1u; }
  rf_block_exscan<NT / 64>(kb, nkb, sh.wsum);
  return !(nkb == 0 || nkb == nband);
}

// Steps 5-6: the nkb band tokens with the best exact scores (sh.band_score) are retained; the ascending index list
// is rewritten from the bitmap if anything changed.
template <int NT>
__device__ void rf_apply(RfShared<NT>& sh, int32_t* __restrict__ out, int N, int nband, int nkb, int kb) {
  if ((int)threadIdx.x < nband) {
    const int keep = band_keeps(sh.band_score, nband, nkb, threadIdx.x);
    sh.keep_new[threadIdx.x] = keep;
    if (keep != kb) sh.s_changed = 1;
  }
  __syncthreads();
  if (!sh.s_changed) return;
  if ((int)threadIdx.x < nband) {
    const int j = sh.band[threadIdx.x];
    if (sh.keep_new[threadIdx.x]) atomicOr(&sh.bitmap[j >> 5], 1u << (j & 31));
    else atomicAnd(&sh.bitmap[j >> 5], ~(1u << (j & 31)));
  }
  __syncthreads();
  const int words = (N + 31) / 32;
  const int wseg = (words + NT - 1) / NT;
  const int w0 = min(words, (int)threadIdx.x * wseg), w1 = min(words, w0 + wseg);
  int pc = 0;
  for (int wi = w0; wi < w1; ++wi) pc += __popc(sh.bitmap[wi]);
  int total;
  int o = rf_block_exscan<NT / 64>(pc, total, sh.wsum);
  for (int wi = w0; wi < w1; ++wi) {
    uint32_t bits = sh.bitmap[wi];
    while (bits) {
      const int bpos = __ffs(bits) - 1;
      bits &= bits - 1;
      out[o++] = wi * 32 + bpos;
    }
  }
}

template <typename T, int NT>
__global__ __launch_bounds__(NT) void k_refine(const T* __restrict__ K, const T* __restrict__ Q,
                                                const float* __restrict__ scores,
                                                const double* __restrict__ row_lse, int N, int d, int R,
                                                int max_budget, int32_t* __restrict__ idx,
                                                const int32_t* __restrict__ n_keep, int scs, int kvs) {
  __shared__ RfShared<NT> sh;
  const int head = blockIdx.x;
  const int n = n_keep[head];
  if (n <= 0 || n >= N) return;
  const float* sc = scores + (size_t)head * scs;
  int32_t* out = idx + (size_t)head * max_budget;
  int nband, nkb, kb;
  if (!rf_find_band<NT>(sh, sc, out, n, N, nband, nkb, kb)) return;
  // 4. exact scores of the band tokens
  rescore_band<T, NT / 64>(K + (size_t)head * kvs * d, Q + (size_t)head * R * d, row_lse + (size_t)head * R, d, R, sh.band,
                           nband, sh.band_score);
  __syncthreads();
  rf_apply<NT>(sh, out, N, nband, nkb, kb);
}

// Layerwise selections (scores, idx, n_keep per layer; K, Q, row_lse per head), in two launches so that the exact
// scores of the band are computed by one workgroup per (layer, head): this one finds the layer's band (the same
// deterministic steps in every workgroup of the layer) and writes the head's exact masses of the band tokens.
template <typename T, int NT>
__global__ __launch_bounds__(NT) void k_refine_layer_part(const T* __restrict__ K, const T* __restrict__ Q,
                                                          const float* __restrict__ layer_scores,
                                                          const double* __restrict__ row_lse, int N, int d, int R, int H,
                                                          int max_budget, const int32_t* __restrict__ idx_layer,
                                                          const int32_t* __restrict__ n_keep_layer,
                                                          double* __restrict__ part /*[L*H][kBandCap]*/, int kvs) {
  __shared__ RfShared<NT> sh;
  const int head = blockIdx.x, l = head / H;
  const int n = n_keep_layer[l];
  if (n <= 0 || n >= N) return;
  int nband, nkb, kb;
  if (!rf_find_band<NT>(sh, layer_scores + (size_t)l * N, idx_layer + (size_t)l * max_budget, n, N, nband, nkb, kb)) return;
  rescore_band<T, NT / 64>(K + (size_t)head * kvs * d, Q + (size_t)head * R * d, row_lse + (size_t)head * R, d, R, sh.band,
                           nband, part + (size_t)head * kBandCap);
}

// Second launch: one workgroup per layer finds the band again, adds the heads' exact masses in head order and
// re-decides the band.
template <int NT>
__global__ __launch_bounds__(NT) void k_refine_layer_apply(const float* __restrict__ layer_scores, int N, int H,
                                                           int max_budget, int32_t* __restrict__ idx_layer,
                                                           const int32_t* __restrict__ n_keep_layer,
                                                           const double* __restrict__ part) {
  __shared__ RfShared<NT> sh;
  const int l = blockIdx.x;
  const int n = n_keep_layer[l];
  if (n <= 0 || n >= N) return;
  int32_t* out = idx_layer + (size_t)l * max_budget;
  int nband, nkb, kb;
  if (!rf_find_band<NT>(sh, layer_scores + (size_t)l * N, out, n, N, nband, nkb, kb)) return;
  if ((int)threadIdx.x < nband) {
    double s = 0.0;
    for (int h = 0; h < H; ++h) s += part[((size_t)l * H + h) * kBandCap + threadIdx.x];
    sh.band_score[threadIdx.x] = s;
  }
  __syncthreads();
  rf_apply<NT>(sh, out, N, nband, nkb, kb);
}

obf_status_t launch_refine(const Dims& m, const Workspace& w, char* ws, const void* K, const void* Q,
                           const float* scores, const double* row_lse, int32_t max_budget, int32_t* idx,
                           const int32_t* n_keep, hipStream_t st) {
  (void)w; (void)ws;
  ProfScope prof_(ST_REFINE, st);
  if (m.dtype == OBF_BF16)
    hipLaunchKernelGGL((k_refine<uint16_t, RF_THREADS>), dim3(m.heads), dim3(RF_THREADS), 0, st, (const uint16_t*)K,
                       (const uint16_t*)Q, scores, row_lse, m.N, m.d, m.R, max_budget, idx, n_keep, m.scs, m.kvs);
  else
    hipLaunchKernelGGL((k_refine<float, RF_THREADS>), dim3(m.heads), dim3(RF_THREADS), 0, st, (const float*)K,
                       (const float*)Q, scores, row_lse, m.N, m.d, m.R, max_budget, idx, n_keep, m.scs, m.kvs);
  return check_launch("refine");
}

// The same re-decision for selections shared by the heads of a layer: scores, idx and n_keep are per layer;
// part is scratch for the heads' exact masses of the band tokens ([L*H][kBandCap] doubles).
obf_status_t launch_refine_layers(const Dims& m, const void* K, const void* Q, const float* layer_scores,
                                  const double* row_lse, int32_t max_budget, int32_t* idx_layer,
                                  const int32_t* n_keep_layer, double* part, hipStream_t st) {
  ProfScope prof_(ST_REFINE, st);
  if (m.dtype == OBF_BF16)
    hipLaunchKernelGGL((k_refine_layer_part<uint16_t, RF_THREADS>), dim3(m.heads), dim3(RF_THREADS), 0, st,
                       (const uint16_t*)K, (const uint16_t*)Q, layer_scores, row_lse, m.N, m.d, m.R, m.H, max_budget,
                       idx_layer, n_keep_layer, part, m.kvs);
  else
    hipLaunchKernelGGL((k_refine_layer_part<float, RF_THREADS>), dim3(m.heads), dim3(RF_THREADS), 0, st,
                       (const float*)K, (const float*)Q, layer_scores, row_lse, m.N, m.d, m.R, m.H, max_budget,
                       idx_layer, n_keep_layer, part, m.kvs);
  if (check_launch("refine (layerwise, exact masses)") != OBF_OK) return OBF_ERR_HIP;
  hipLaunchKernelGGL((k_refine_layer_apply<RF_THREADS>), dim3(m.L), dim3(RF_THREADS), 0, st, layer_scores, m.N, m.H,
                     max_budget, idx_layer, n_keep_layer, part);
  return check_launch("refine (layerwise)");
}

}  // namespace obf
