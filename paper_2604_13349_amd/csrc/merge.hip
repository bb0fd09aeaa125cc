// The cache-merging comparison system of App. E on an already selected and gathered head:
//   (ii)  route every deleted token j to the retained slot whose key has the highest cosine similarity with K_j
//         (the first maximum wins; a key of zero norm has cosine 0 with everything);
//   (iii) V*_t = V_t + sum over the deleted j routed to t of A_j / (A_t + eps) V_j; keys unchanged.
// Step (i) is the library's TopK_B.  The routing is a (tokens x slots x head_dim) contraction: bf16 caches with
// head_dim 128 run it on the matrix cores (exact bf16 products, fp32 accumulation), other shapes on the vector ALU in
// fp32.  The cosine of token j with slot t is <K_j, K_t> / (|K_j| |K_t|); 1 / |K_j| is the same for every slot, so the
// arg-max only needs <K_j, K_t> / |K_t| (sign and order preserved), and an all-zero K_j routes to slot 0.
#include "common.hpp"

namespace obf {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int MG_THREADS = 256;
constexpr int MG_D = 128;
constexpr int MG_KK = MG_D / 16;
constexpr int MG_SLOTS_PER_WAVE = 8;     // merge: retained slots whose sums one wave carries
constexpr int MG_SLOTS_PER_WG = 4 * MG_SLOTS_PER_WAVE;

union MgFrag { uint4 u; bf16x8 v; };

// 1 / |K_t| of every retained key (0 for a zero key), from the gathered keys: one wave per slot.
template <typename T>
__global__ __launch_bounds__(MG_THREADS) void k_mg_inv_norm(const T* __restrict__ K_out, const int32_t* __restrict__ n_keep,
                                                            int d, int max_budget, float* __restrict__ inv_norm) {
  const int head = blockIdx.y, lane = threadIdx.x & 63;
  const int slot = blockIdx.x * (MG_THREADS / 64) + (threadIdx.x >> 6);
  if (slot >= max_budget) return;
  float s = 0.f;
  if (slot < n_keep[head]) {
    const T* row = K_out + ((size_t)head * max_budget + slot) * d;
    for (int c = lane; c < d; c += 64) { const float x = Elem<T>::load(row + c); s = fmaf(x, x, s); }
  }
  for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
  if (lane == 0) inv_norm[(size_t)head * max_budget + slot] = s > 0.f ? 1.0f / sqrtf(s) : 0.f;
}

// Routing on the matrix cores.  One wave owns 32 tokens (lane l and lane l + 32 both hold token l % 32, the two halves
// of head_dim's 16-element MFMA steps); it walks the retained slots 32 at a time: the 32 x 32 tile of dot products has,
// in entry i of lane l, slot s0 + (i/4)*8 + (l/32)*4 + i%4 against token l%32, so the running maximum is kept per lane
// over slots in ascending order and the two lanes of a token are combined at the end.
__global__ __launch_bounds__(MG_THREADS) void k_mg_route_mfma(const uint16_t* __restrict__ K, const uint16_t* __restrict__ K_out,
                                                              const float* __restrict__ inv_norm,
                                                              const int32_t* __restrict__ n_keep, int N, int kvs,
                                                              int max_budget, int32_t* __restrict__ route) {
  const int head = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lr = lane & 31, lh = lane >> 5;
  const int tok = blockIdx.x * 128 + wave * 32 + lr;
  const int nk = n_keep[head];
  int32_t* rt = route + (size_t)head * N;
  if (nk <= 0) { if (lh == 0 && tok < N) rt[tok] = -1; return; }
  const uint16_t* Kh = K + (size_t)head * kvs * MG_D;
  const uint16_t* Ko = K_out + (size_t)head * max_budget * MG_D;
  const float* inv = inv_norm + (size_t)head * max_budget;
  MgFrag tf[MG_KK];
  {
    const uint4* p = (const uint4*)(Kh + (size_t)min(tok, N - 1) * MG_D + lh * 8);
#pragma unroll
    for (int kk = 0; kk < MG_KK; ++kk) tf[kk].u = p[kk * 2];
  }
  float best = -INFINITY;
  int bslot = 0;
  MgFrag sf[2][MG_KK];
  auto load_slots = [&](MgFrag (&dst)[MG_KK], int s0) {
    const uint4* p = (const uint4*)(Ko + (size_t)min(s0 + lr, nk - 1) * MG_D + lh * 8);      // rows past the list: clamped, masked below
#pragma unroll
    for (int kk = 0; kk < MG_KK; ++kk) dst[kk].u = p[kk * 2];
  };
  load_slots(sf[0], 0);
  int buf = 0;
  for (int s0 = 0; s0 < nk; s0 += 32, buf ^= 1) {
    if (s0 + 32 < nk) load_slots(sf[buf ^ 1], s0 + 32);
    f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < MG_KK; ++kk) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sf[buf][kk].v, tf[kk].v, acc, 0, 0, 0);
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {
      const int sb = s0 + i4 * 8 + lh * 4;                      // this lane's four consecutive slots of the group
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int s = sb + e;
        if (s < nk) {
          const float c = acc[i4 * 4 + e] * inv[s];
          if (c > best) { best = c; bslot = s; }               // strict: the first maximum wins
        }
      }
    }
  }
  const float ob = __shfl_xor(best, 32);
  const int os = __shfl_xor(bslot, 32);
  if (ob > best || (ob == best && os < bslot)) { best = ob; bslot = os; }
  if (lh == 0 && tok < N) rt[tok] = bslot;
}

// Routing on the vector ALU (fp32 caches, head_dim 64): one thread per token, the retained keys staged through LDS
// 32 at a time; fp32 products and sums.
template <typename T>
__global__ __launch_bounds__(MG_THREADS) void k_mg_route_generic(const T* __restrict__ K, const T* __restrict__ K_out,
                                                                 const float* __restrict__ inv_norm,
                                                                 const int32_t* __restrict__ n_keep, int N, int d, int kvs,
                                                                 int max_budget, int32_t* __restrict__ route) {
  __shared__ float ks[32][129];
  const int head = blockIdx.y;
  const int tok = blockIdx.x * MG_THREADS + threadIdx.x;
  const int nk = n_keep[head];
  int32_t* rt = route + (size_t)head * N;
  if (nk <= 0) { if (tok < N) rt[tok] = -1; return; }
  const T* kr = K + ((size_t)head * kvs + min(tok, N - 1)) * d;
  const T* Ko = K_out + (size_t)head * max_budget * d;
  const float* inv = inv_norm + (size_t)head * max_budget;
  float best = -INFINITY;
  int bslot = 0;
  for (int s0 = 0; s0 < nk; s0 += 32) {
    __syncthreads();
    for (int e = threadIdx.x; e < 32 * d; e += MG_THREADS) {
      const int r = e / d, c = e % d;
      ks[r][c] = (s0 + r < nk) ? Elem<T>::load(Ko + (size_t)(s0 + r) * d + c) : 0.f;
    }
    __syncthreads();
    const int ns = min(32, nk - s0);
    for (int r = 0; r < ns; ++r) {
      float acc = 0.f;
      for (int c = 0; c < d; ++c) acc = fmaf(Elem<T>::load(kr + c), ks[r][c], acc);
      const float cs = acc * inv[s0 + r];
      if (cs > best) { best = cs; bslot = s0 + r; }
    }
  }
  if (tok < N) rt[tok] = bslot;
}

__global__ __launch_bounds__(MG_THREADS) void k_mg_fill(int32_t* __restrict__ p, size_t n, int32_t v) {
  const size_t i = (size_t)blockIdx.x * MG_THREADS + threadIdx.x;
  if (i < n) p[i] = v;
}

// retained tokens take no part in the routing
__global__ __launch_bounds__(MG_THREADS) void k_mg_unroute_kept(const int32_t* __restrict__ idx, const int32_t* __restrict__ n_keep,
                                                                int N, int max_budget, int32_t* __restrict__ route) {
  const int head = blockIdx.y;
  const int t = blockIdx.x * MG_THREADS + threadIdx.x;
  if (t < n_keep[head] && t < max_budget) route[(size_t)head * N + idx[(size_t)head * max_budget + t]] = -1;
}

// The same per-slot sums serve the Per-token alternative of App. D (PER_TOKEN; the reading: the deleted tokens are shared
// out among the slots by the routing above, slot t's direction is B a_del / (a_keep + eps) times the projection of
// sum_{pi(j) = t} A_j v_j / (a_del + eps) onto the residual subspace C of Eq. 5 - C's rows lie in the complement of
// the retained span, so projecting the values is projecting their residuals; the mean over the slots is Eq. 6's delta).
// There the weights are the attention masses themselves, the sums are projected with the k_used rows of C that the
// back-fill kernel left in the head's scratch, and the result is added to the slot's value.
//
// Merge.  A workgroup owns 32 consecutive retained slots, a wave eight of them.  Every wave scans the head's route list
// 64 tokens at a time and, for each token routed to one of its slots, in ascending token order, adds the weighted value
// row into that slot's running sum (LDS, one lane per pair of columns): the order of the additions is fixed, so the
// result is the same on every run.  Slots that received nothing are left as the bit copies the gather wrote.
template <typename T, bool PER_TOKEN>
__global__ __launch_bounds__(MG_THREADS) void k_mg_merge(const T* __restrict__ V, const float* __restrict__ scores,
                                                         const int32_t* __restrict__ idx, const int32_t* __restrict__ n_keep,
                                                         const int32_t* __restrict__ route, int N, int d, int kvs, int scs,
                                                         int max_budget, T* __restrict__ V_out,
                                                         const HeadState* __restrict__ state /*PER_TOKEN*/,
                                                         const float* __restrict__ mats /*PER_TOKEN: [heads][3][d*d], C in the second matrix*/,
                                                         int no_scaling) {
  __shared__ float acc[4][MG_SLOTS_PER_WAVE][MG_D];
  __shared__ float a_slot[4][MG_SLOTS_PER_WAVE];
  __shared__ int cnt[4][MG_SLOTS_PER_WAVE];
  __shared__ float cb[PER_TOKEN ? 16 : 1][MG_D];               // the rows of C
  const int head = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nk = min(n_keep[head], max_budget);
  int kc = 0;
  float pt_scale = 0.f;
  if (PER_TOKEN) {
    const HeadState hs = state[head];
    if (!hs.active || hs.k_used <= 0) return;                  // no injection for this head (uniform over the workgroup)
    kc = min(hs.k_used, 16);
    const float* Cg = mats + ((size_t)head * 3 + 1) * d * d;
    for (int e = threadIdx.x; e < kc * d; e += MG_THREADS) cb[e / d][e % d] = Cg[e];
    pt_scale = (float)((double)hs.n_keep * (no_scaling ? 1.0 : hs.a_del / (hs.a_keep + kEps)) / (hs.a_del + kEps));
    __syncthreads();
  }
  const int slot0 = blockIdx.x * MG_SLOTS_PER_WG + wave * MG_SLOTS_PER_WAVE;
  if (slot0 >= nk) return;                                     // whole wave: nothing to own (no barrier below)
  const float* sc = scores + (size_t)head * scs;
  const int32_t* rt = route + (size_t)head * N;
  const T* Vh = V + (size_t)head * kvs * d;
  for (int e = lane; e < MG_SLOTS_PER_WAVE * MG_D; e += 64) acc[wave][e / MG_D][e % MG_D] = 0.f;
  if (lane < MG_SLOTS_PER_WAVE) {
    cnt[wave][lane] = 0;
    a_slot[wave][lane] = (slot0 + lane < nk) ? sc[idx[(size_t)head * max_budget + slot0 + lane]] : 0.f;
  }
  __builtin_amdgcn_wave_barrier();
  for (int base = 0; base < N; base += 64) {
    const int j = base + lane;
    const int r = (j < N) ? rt[j] : -1;
    const unsigned local = (unsigned)(r - slot0);
    uint64_t mask = __ballot(r >= 0 && local < (unsigned)MG_SLOTS_PER_WAVE);
    while (mask) {
      const int l = __builtin_ctzll(mask);
      mask &= mask - 1;
      const int sl = __shfl((int)local, l);
      const int jj = base + l;
      const float w = PER_TOKEN ? sc[jj] : (float)((double)sc[jj] / ((double)a_slot[wave][sl] + kEps));
      const T* vr = Vh + (size_t)jj * d;
      for (int c = lane; c < d; c += 64) acc[wave][sl][c] = fmaf(w, Elem<T>::load(vr + c), acc[wave][sl][c]);
      if (lane == 0) cnt[wave][sl] += 1;
    }
  }
  __builtin_amdgcn_wave_barrier();
  for (int sl = 0; sl < MG_SLOTS_PER_WAVE; ++sl) {
    if (slot0 + sl >= nk || cnt[wave][sl] == 0) continue;
    T* o = V_out + ((size_t)head * max_budget + slot0 + sl) * d;
    if (PER_TOKEN) {
      // lane l holds columns l and l + 64 of the slot's sum; its coefficient on every row of C, then the combination
      const float u0 = (lane < d) ? acc[wave][sl][lane] : 0.f, u1 = (lane + 64 < d) ? acc[wave][sl][lane + 64] : 0.f;
      float d0 = 0.f, d1 = 0.f;
      for (int i = 0; i < kc; ++i) {
        const float c0 = (lane < d) ? cb[i][lane] : 0.f, c1 = (lane + 64 < d) ? cb[i][lane + 64] : 0.f;
        float g = fmaf(u0, c0, u1 * c1);
        for (int off = 32; off > 0; off >>= 1) g += __shfl_xor(g, off);
        d0 = fmaf(g, c0, d0); d1 = fmaf(g, c1, d1);
      }
      if (lane < d) Elem<T>::store(o + lane, fmaf(pt_scale, d0, Elem<T>::load(o + lane)));
      if (lane + 64 < d) Elem<T>::store(o + lane + 64, fmaf(pt_scale, d1, Elem<T>::load(o + lane + 64)));
    } else {
      for (int c = lane; c < d; c += 64) Elem<T>::store(o + c, Elem<T>::load(o + c) + acc[wave][sl][c]);
    }
  }
}

// steps (ii) and (iii); per_token: the per-slot directions of App. D's Per-token alternative instead of the merge
static obf_status_t run_merge(const Dims& m, const Workspace& w, char* ws, const void* K, const void* V, const float* scores,
                              const int32_t* idx, const int32_t* n_keep, int32_t max_budget, const void* K_out,
                              void* V_out, int32_t* route_out, hipStream_t st, bool per_token, int no_scaling) {
  const HeadState* state = (const HeadState*)(ws + w.head_state);
  const float* mats = (const float*)(ws + w.mats);
  if (max_budget == 0) {                                         // nothing retained: nothing to route to
    if (route_out) {
      const size_t n = (size_t)m.heads * m.N;
      hipLaunchKernelGGL(k_mg_fill, dim3((unsigned)((n + MG_THREADS - 1) / MG_THREADS)), dim3(MG_THREADS), 0, st, route_out, n, -1);
      return check_launch("merge fill");
    }
    return OBF_OK;
  }
  float* inv_norm = (float*)(ws + w.inv_norm);
  int32_t* route = route_out ? route_out : (int32_t*)(ws + w.route);
  const bool bf = m.dtype == OBF_BF16;
  dim3 gn((max_budget + 3) / 4, m.heads);
  if (bf) hipLaunchKernelGGL(k_mg_inv_norm<uint16_t>, gn, dim3(MG_THREADS), 0, st, (const uint16_t*)K_out, n_keep, m.d, max_budget, inv_norm);
  else hipLaunchKernelGGL(k_mg_inv_norm<float>, gn, dim3(MG_THREADS), 0, st, (const float*)K_out, n_keep, m.d, max_budget, inv_norm);
  if (check_launch("merge inv_norm") != OBF_OK) return OBF_ERR_HIP;
  if (bf && m.d == MG_D) {
    hipLaunchKernelGGL(k_mg_route_mfma, dim3((m.N + 127) / 128, m.heads), dim3(MG_THREADS), 0, st, (const uint16_t*)K,
                       (const uint16_t*)K_out, inv_norm, n_keep, m.N, m.kvs, max_budget, route);
  } else if (bf) {
    hipLaunchKernelGGL(k_mg_route_generic<uint16_t>, dim3((m.N + MG_THREADS - 1) / MG_THREADS, m.heads), dim3(MG_THREADS), 0, st,
                       (const uint16_t*)K, (const uint16_t*)K_out, inv_norm, n_keep, m.N, m.d, m.kvs, max_budget, route);
  } else {
    hipLaunchKernelGGL(k_mg_route_generic<float>, dim3((m.N + MG_THREADS - 1) / MG_THREADS, m.heads), dim3(MG_THREADS), 0, st,
                       (const float*)K, (const float*)K_out, inv_norm, n_keep, m.N, m.d, m.kvs, max_budget, route);
  }
  if (check_launch("merge route") != OBF_OK) return OBF_ERR_HIP;
  hipLaunchKernelGGL(k_mg_unroute_kept, dim3((max_budget + MG_THREADS - 1) / MG_THREADS, m.heads), dim3(MG_THREADS), 0, st, idx,
                     n_keep, m.N, max_budget, route);
  if (check_launch("merge unroute") != OBF_OK) return OBF_ERR_HIP;
  dim3 gm((max_budget + MG_SLOTS_PER_WG - 1) / MG_SLOTS_PER_WG, m.heads);
#define OBF_MG_LAUNCH(T, PT) hipLaunchKernelGGL((k_mg_merge<T, PT>), gm, dim3(MG_THREADS), 0, st, (const T*)V, scores, idx, n_keep, \
                                               route, m.N, m.d, m.kvs, m.scs, max_budget, (T*)V_out, state, mats, no_scaling)
  if (bf && per_token) OBF_MG_LAUNCH(uint16_t, true);
  else if (bf) OBF_MG_LAUNCH(uint16_t, false);
  else if (per_token) OBF_MG_LAUNCH(float, true);
  else OBF_MG_LAUNCH(float, false);
#undef OBF_MG_LAUNCH
  return check_launch("merge values");
}

obf_status_t launch_cache_merge(const Dims& m, const Workspace& w, char* ws, const void* K, const void* V, const float* scores,
                                const int32_t* idx, const int32_t* n_keep, int32_t max_budget, const void* K_out,
                                void* V_out, int32_t* route_out, hipStream_t st) {
  return run_merge(m, w, ws, K, V, scores, idx, n_keep, max_budget, K_out, V_out, route_out, st, false, 0);
}

obf_status_t launch_per_token_inject(const Dims& m, const Workspace& w, char* ws, const void* K, const void* V,
                                     const float* scores, const int32_t* idx, const int32_t* n_keep, int32_t max_budget,
                                     const void* K_out, void* V_out, int no_scaling, hipStream_t st) {
  if (m.d > MG_D) { set_error("per-token variant: head_dim above 128"); return OBF_ERR_UNSUPPORTED; }
  return run_merge(m, w, ws, K, V, scores, idx, n_keep, max_budget, K_out, V_out, nullptr, st, true, no_scaling);
}

}  // namespace obf
