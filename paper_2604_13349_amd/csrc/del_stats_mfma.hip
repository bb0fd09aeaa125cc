// Statistics of the deleted value rows of a head, for the residual of Eq. 3 - 4, on the matrix cores (bf16 caches,
// head_dim 128): per chunk of 1024 tokens the partial Gram V_del^T V_del (products of bf16 values are exact in fp32,
// accumulation is fp32), the weighted sum  sum_j A_j v_j  and  sum_j ||v_j||^2  over the deleted rows of the chunk.
// Retained rows enter as zeros.  Output format and meaning are those of the reference-precision kernel it replaces:
// gram_part[head][chunk] = { G [d][d], u [d], ||V_del||^2, pad[3] }.
#include "common.hpp"

namespace obf {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 dm_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float dm_f32x16;

constexpr int DM_THREADS = 256;
constexpr int DM_D = 128;
constexpr int DM_TILE = 64;              // rows staged per iteration
constexpr int DM_LDW = 136;              // staging stride in 32-bit words per token PAIR
static_assert(kStatChunk % DM_TILE == 0, "a chunk is a whole number of tiles");

union DmFrag { uint32_t w[4]; dm_bf16x8 v; };

// The lower triangle of G is ten 32x32 tiles (row block rb >= column block cb), three or two per wave; entry i of
// lane l of a tile is G[rb*32 + (i/4)*8 + (l/32)*4 + (i%4)][cb*32 + l%32].
__device__ __forceinline__ void dm_wave_tiles(int wave, int (&rb)[3], int (&cb)[3], int& nt) {
  if (wave == 0) { rb[0] = 0; cb[0] = 0; rb[1] = 1; cb[1] = 1; rb[2] = 3; cb[2] = 2; nt = 3; }
  else if (wave == 1) { rb[0] = 1; cb[0] = 0; rb[1] = 2; cb[1] = 1; rb[2] = 3; cb[2] = 3; nt = 3; }
  else if (wave == 2) { rb[0] = 2; cb[0] = 0; rb[1] = 3; cb[1] = 1; rb[2] = 0; cb[2] = 0; nt = 2; }
  else { rb[0] = 3; cb[0] = 0; rb[1] = 2; cb[1] = 2; rb[2] = 0; cb[2] = 0; nt = 2; }
}

// One chunk of one head (the whole workgroup).
__device__ __forceinline__ void dm_chunk(const uint16_t* __restrict__ V, const float* __restrict__ scores,
                                         const int32_t* __restrict__ idx, int N, int max_budget, int nstat,
                                         const HeadState* __restrict__ state, const int32_t* __restrict__ n_keep,
                                         float* __restrict__ gram_part, int scs, int kvs, int head, int chunk) {
  const int n = n_keep ? n_keep[head] : state[head].n_keep;
  if (n_keep ? !(n > 0 && n < N) : !state[head].active) return;
  __shared__ uint32_t stage[2][(DM_TILE / 2) * DM_LDW];
  __shared__ float wt[kStatChunk];                     // score of a deleted token of the chunk, 0 for a retained one
  __shared__ uint32_t kept[kStatChunk / 32];           // bitmap of the retained tokens of the chunk
  __shared__ float red[8][DM_D + 1];                   // cross-thread reduction of u and ||.||^2
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lr = lane & 31, lh = lane >> 5;
  const int32_t* id = idx + (size_t)head * max_budget;
  const uint16_t* Vh = V + (size_t)head * kvs * DM_D;
  const float* sc = scores + (size_t)head * scs;
  const int t0 = chunk * kStatChunk, t1 = min(N, t0 + kStatChunk);
  const int rows = t1 - t0;

  // which tokens of the chunk are retained; weights
  for (int i = tid; i < kStatChunk / 32; i += DM_THREADS) kept[i] = 0u;
  __syncthreads();
  for (int i = tid; i < n; i += DM_THREADS) {
    const int j = id[i] - t0;
    if (j >= 0 && j < rows) atomicOr(&kept[j >> 5], 1u << (j & 31));
  }
  __syncthreads();
  for (int i = tid; i < kStatChunk; i += DM_THREADS) {
    const bool del = i < rows && !((kept[i >> 5] >> (i & 31)) & 1u);
    wt[i] = del ? sc[t0 + i] : 0.f;
  }
  // (visible to everyone after the first barrier of the pipeline below)

  int trb[3], tcb[3], nt;
  dm_wave_tiles(wave, trb, tcb, nt);
  dm_f32x16 acc[3];
#pragma unroll
  for (int t = 0; t < 3; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;
  float u4[4] = {0.f, 0.f, 0.f, 0.f};                  // weighted sums of this thread's four columns 4*(tid%32) ..
  float s4[4] = {0.f, 0.f, 0.f, 0.f};                  // plain sums of the same columns (deleted rows only)
  float nn = 0.f;                                      // squared norms of the deleted entries this thread has seen

  uint2 pre[2][8];
  auto fetch = [&](uint2 (&dst)[8], int r0) {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int e = tid + q * DM_THREADS;
      const int r = r0 + (e >> 5), c = e & 31;
      dst[q] = make_uint2(0u, 0u);
      if (r < rows) dst[q] = *(const uint2*)(Vh + (size_t)(t0 + r) * DM_D + c * 4);
    }
  };
  // Staging layout: word [p][j] holds column j of tokens 2p and 2p+1 (low / high half), so that an operand fragment
  // (8 tokens of one column) is four 32-bit reads.  Lanes l and l+32 of a wave hold rows 2p and 2p+1 of the same four
  // columns; the lower lane writes the words of the first two, the upper lane of the last two.  Retained rows are
  // zeroed here, and the weighted sum and the squared norm are taken from the same registers.
  auto put = [&](const uint2 (&src)[8], int buf, int r0) {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int e = tid + q * DM_THREADS;
      const int r = r0 + (e >> 5);
      const int pr = e >> 6, c = e & 31;
      const float w = (r < rows) ? wt[r] : 0.f;
      const bool del = (r < rows) && !((kept[r >> 5] >> (r & 31)) & 1u);
      const uint32_t sx = del ? src[q].x : 0u, sy = del ? src[q].y : 0u;
      {
        const float v0 = __uint_as_float(sx << 16), v1 = __uint_as_float(sx & 0xffff0000u);
        const float v2 = __uint_as_float(sy << 16), v3 = __uint_as_float(sy & 0xffff0000u);
        u4[0] = fmaf(w, v0, u4[0]); u4[1] = fmaf(w, v1, u4[1]); u4[2] = fmaf(w, v2, u4[2]); u4[3] = fmaf(w, v3, u4[3]);
        s4[0] += v0; s4[1] += v1; s4[2] += v2; s4[3] += v3;
        nn = fmaf(v0, v0, nn); nn = fmaf(v1, v1, nn); nn = fmaf(v2, v2, nn); nn = fmaf(v3, v3, nn);
      }
      const uint32_t mine = lh ? sy : sx;
      const uint32_t other = lh ? sx : sy;
      const auto sw = __builtin_amdgcn_permlane32_swap(other, other, false, false);
      const uint32_t theirs = lh ? sw[0] : sw[1];
      const uint32_t even = lh ? theirs : mine, odd = lh ? mine : theirs;     // rows 2p and 2p+1
      uint2 wv;
      wv.x = (even & 0xffffu) | (odd << 16);
      wv.y = (even >> 16) | (odd & 0xffff0000u);
      *(uint2*)(&stage[buf][pr * DM_LDW + c * 4 + lh * 2]) = wv;
    }
  };
  auto compute = [&](const uint32_t* st) {
#pragma unroll
    for (int ks = 0; ks < DM_TILE / 16; ++ks) {
      DmFrag f[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint32_t* p = st + (ks * 8 + lh * 4) * DM_LDW + c * 32 + lr;
#pragma unroll
        for (int i = 0; i < 4; ++i) f[c].w[i] = p[i * DM_LDW];
      }
      if (wave == 0) {
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[0].v, f[0].v, acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[1].v, f[1].v, acc[1], 0, 0, 0);
        acc[2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[3].v, f[2].v, acc[2], 0, 0, 0);
      } else if (wave == 1) {
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[1].v, f[0].v, acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[2].v, f[1].v, acc[1], 0, 0, 0);
        acc[2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[3].v, f[3].v, acc[2], 0, 0, 0);
      } else if (wave == 2) {
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[2].v, f[0].v, acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[3].v, f[1].v, acc[1], 0, 0, 0);
      } else {
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[3].v, f[0].v, acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[2].v, f[2].v, acc[1], 0, 0, 0);
      }
    }
  };
  fetch(pre[0], 0);
  fetch(pre[1], DM_TILE);
  __syncthreads();                       // wt and kept complete
  put(pre[0], 0, 0);
  fetch(pre[0], 2 * DM_TILE);
  __syncthreads();
  for (int r0 = 0; r0 < rows; r0 += 2 * DM_TILE) {
    // even tile: in stage[0]; pre[1] holds tile r0+64, pre[0] holds tile r0+128
    compute(stage[0]);
    put(pre[1], 1, r0 + DM_TILE);
    fetch(pre[1], r0 + 3 * DM_TILE);
    __syncthreads();
    if (r0 + DM_TILE < rows) compute(stage[1]);
    put(pre[0], 0, r0 + 2 * DM_TILE);
    fetch(pre[0], r0 + 4 * DM_TILE);
    __syncthreads();
  }

  // ---- results: the 32 x 32 tiles of the Gram matrix on and below the diagonal (row-major in the d x d partial, so
  // the stores are row segments; the tiles above the diagonal are left unwritten, the reader mirrors)
  float* out = gram_part + ((size_t)head * nstat + chunk) * gram_stride(DM_D);
#pragma unroll
  for (int t = 0; t < 3; ++t) {
    if (t < nt) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int row = trb[t] * 32 + (i >> 2) * 8 + lh * 4 + (i & 3), col = tcb[t] * 32 + lr;
        out[row * DM_D + col] = acc[t][i];
      }
    }
  }
  // ---- weighted sum and squared norm: the eight threads with the same tid % 32 own the same four columns
  {
    const int c = tid & 31, part = tid >> 5;
#pragma unroll
    for (int k = 0; k < 4; ++k) red[part][c * 4 + k] = u4[k];
    // squared norms: wave-level sum first (fixed order), then the four waves
    float s = nn;
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
    if (lane == 0) red[wave][DM_D] = s;
  }
  __syncthreads();
  if (tid < DM_D) {
    float s = 0.f;
#pragma unroll
    for (int p = 0; p < 8; ++p) s += red[p][tid];
    out[DM_D * DM_D + tid] = s;
  }
  if (tid == 0) out[DM_D * DM_D + 2 * DM_D] = (red[0][DM_D] + red[1][DM_D]) + (red[2][DM_D] + red[3][DM_D]);
  __syncthreads();
  {
    const int c = tid & 31, part = tid >> 5;
#pragma unroll
    for (int k = 0; k < 4; ++k) red[part][c * 4 + k] = s4[k];
  }
  __syncthreads();
  if (tid < DM_D) {
    float s = 0.f;
#pragma unroll
    for (int p = 0; p < 8; ++p) s += red[p][tid];
    out[DM_D * DM_D + DM_D + tid] = s;
  }
}

// The active head whose number (in head order) is `target`, or -1; every thread gets it.  s_i has 5 entries.
__device__ int dm_active_head(const HeadState* __restrict__ state, int heads, int target, int* s_i) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (threadIdx.x == 0) s_i[4] = -1;
  int base = 0;
  for (int h0 = 0; h0 < heads; h0 += DM_THREADS) {
    const int h = h0 + threadIdx.x;
    const bool p = h < heads && state[h].active != 0;
    const uint64_t mask = __ballot(p);
    __syncthreads();
    if (lane == 0) s_i[wave] = __popcll(mask);
    __syncthreads();
    int before = base, tot = 0;
    for (int w = 0; w < DM_THREADS / 64; ++w) { if (w < wave) before += s_i[w]; tot += s_i[w]; }
    if (p && before + __popcll(mask & ((1ull << lane) - 1ull)) == target) s_i[4] = h;
    base += tot;
    if (base > target) break;                        // uniform: found
  }
  __syncthreads();
  return s_i[4];
}

// grid (chunks, heads): workgroup (c, h) takes chunk c of head h.  With compact != 0 the grid is (chunks, a few rows) and
// row y takes the active heads number y, y + rows, ... (found by scanning the head states): for calls in which the
// certificate settles nearly every head, so that a launch over all heads would consist of workgroups that exit at once.
__global__ __launch_bounds__(DM_THREADS, 2) void k_bf_del_stats_mfma(const uint16_t* __restrict__ V,
                                                                     const float* __restrict__ scores,
                                                                     const int32_t* __restrict__ idx, int N,
                                                                     int max_budget, int nstat,
                                                                     const HeadState* __restrict__ state,
                                                                     const int32_t* __restrict__ n_keep /*non-null: the head states are still being written; every head with deleted rows is active*/,
                                                                     float* __restrict__ gram_part, int scs, int kvs,
                                                                     int compact, int heads) {
  if (!compact) {
    dm_chunk(V, scores, idx, N, max_budget, nstat, state, n_keep, gram_part, scs, kvs, blockIdx.y, blockIdx.x);
    return;
  }
  __shared__ int s_i[5];
  for (int s = blockIdx.y;; s += gridDim.y) {
    const int head = dm_active_head(state, heads, s, s_i);
    if (head < 0) return;
    dm_chunk(V, scores, idx, N, max_budget, nstat, state, n_keep, gram_part, scs, kvs, head, blockIdx.x);
  }
}

bool del_stats_mfma_supported(const Dims& m) { return m.dtype == OBF_BF16 && m.d == DM_D; }

obf_status_t launch_del_stats_mfma(const Dims& m, const Workspace& w, const void* V, const float* scores,
                                   const int32_t* idx, int32_t max_budget, const HeadState* state,
                                   const int32_t* n_keep, float* gram_part, hipStream_t st, bool few_active) {
  // few_active: the head states are final (n_keep == nullptr) and nearly all heads are expected to be inactive
  // (a launch of a few thousand workgroups that exit at once is still cheaper than the scan)
  const int compact = (few_active && !n_keep && (long)w.nstat * m.heads >= 4096) ? 1 : 0;
  { ProfScope prof_(ST_DEL_STATS, st);
    hipLaunchKernelGGL(k_bf_del_stats_mfma, dim3(w.nstat, compact ? 8 : m.heads), dim3(DM_THREADS), 0, st, (const uint16_t*)V,
                       scores, idx, m.N, max_budget, w.nstat, state, n_keep, gram_part, m.scs, m.kvs, compact, m.heads); }
  return check_launch("backfill del_stats (mfma)");
}

}  // namespace obf
