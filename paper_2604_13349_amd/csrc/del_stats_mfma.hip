// Statistics of the deleted value rows of a head, for the residual of Eq. 3 - 4, on the matrix cores (bf16 caches,
// head_dim 128): per chunk of 1024 tokens the partial Gram V_del^T V_del (products of bf16 values are exact in fp32,
// accumulation is fp32), the weighted sum  sum_j A_j v_j,  the plain sum  sum_j v_j  and  sum_j ||v_j||^2  over the
// deleted rows of the chunk.  Retained rows enter as zeros.  The two sums are matrix products as well: the weight of
// a token, split into three bf16 parts that add up to it exactly, and the constant one are four more "columns" next
// to the 128 value columns, and the squared norm is the trace of the Gram matrix - the vector ALU only moves data.
// Output format and meaning are those of the reference-precision kernel it replaces:
// gram_part[head][chunk] = { G [d][d], u [d], s [d], ||V_del||^2, pad[3] }.
#include "common.hpp"
#include "gram_stage.hpp"
#include "wave_ops.hpp"

namespace obf {

typedef gs_f32x16 dm_f32x16;

constexpr int DM_THREADS = 512;
constexpr int DM_WAVES = DM_THREADS / 64;
constexpr int DM_D = GS_D;
constexpr int DM_TILE = GS_TILE;         // rows staged per iteration
constexpr int DM_WQ = kStatChunk + 8;    // stride of the weight-part arrays (bf16 entries)
static_assert(kStatChunk % DM_TILE == 0, "a chunk is a whole number of tiles");

typedef GsFrag DmFrag;

// The lower triangle of G is ten 32x32 tiles (row block rb >= column block cb), and the two sums take four more tile
// products (one per 32-column block; such a tile has the weight parts in rows 0 - 2 and the plain sum in row 3, i.e.
// entries 0 - 3 of lanes 0 - 31).  Entry i of lane l of a tile is G[rb*32 + (i/4)*8 + (l/32)*4 + (i%4)][cb*32 + l%32].
// Eight waves, one instruction stream: wave w takes the k-steps 2h, 2h + 1 of every staged tile (h = w / 4: the two
// halves of the workgroup split the tokens, their accumulators meet in LDS at the end) and, with j = w % 4, four
// products per step, the operands picked by LDS address, not by branch:
//   tile (j, 0),  tiles (a, b) and (c, b),  sums of columns 32 j .. 32 j + 31
//   j = 0: (1,1) (2,1)    j = 1: (3,1)    j = 2: (2,2) (3,2)    j = 3: (3,3)
// (j = 1 and j = 3 have one tile less: their third product repeats the second and is dropped).
struct DmTiles { int a, c, b, third; };
__device__ __forceinline__ DmTiles dm_wave_tiles(int j) {
  DmTiles t;
  t.a = (j == 0) ? 1 : (j == 2) ? 2 : 3;
  t.c = (j == 0) ? 2 : 3;
  t.b = (j < 2) ? 1 : j;
  t.third = (j == 0 || j == 2) ? 1 : 0;
  return t;
}
constexpr int DM_NACC = 4;

// One chunk of one head (the whole workgroup).
__device__ __forceinline__ void dm_chunk(const uint16_t* __restrict__ V, const float* __restrict__ scores,
                                         const int32_t* __restrict__ idx, int N, int max_budget, int nstat,
                                         const HeadState* __restrict__ state, const int32_t* __restrict__ n_keep,
                                         float* __restrict__ gram_part, int scs, int kvs, int head, int chunk) {
  const int n = n_keep ? n_keep[head] : state[head].n_keep;
  if (n_keep ? !(n > 0 && n < N) : !state[head].active) return;
  __shared__ __attribute__((aligned(16))) uint32_t stage[2][GS_STAGE_WORDS];
  __shared__ __attribute__((aligned(16))) uint16_t wq[4][DM_WQ];   // bf16: three parts of a deleted token's score, and one; 0 for a retained token
  __shared__ uint32_t kept[kStatChunk / 32];           // bitmap of the retained tokens of the chunk
  __shared__ float red[DM_WAVES];                      // the waves' shares of the trace
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lr = lane & 31, lh = lane >> 5;
  const int32_t* id = idx + (size_t)head * max_budget;
  const uint16_t* Vh = V + (size_t)head * kvs * DM_D;
  const float* sc = scores + (size_t)head * scs;
  const int t0 = chunk * kStatChunk, t1 = min(N, t0 + kStatChunk);
  const int rows = t1 - t0;

  // which tokens of the chunk are retained; weights
  __syncthreads();                                     // a workgroup that takes several heads in turn: the last one is done
  for (int i = tid; i < kStatChunk / 32; i += DM_THREADS) kept[i] = 0u;
  __syncthreads();
  for (int i = tid; i < n; i += DM_THREADS) {
    const int j = id[i] - t0;
    if (j >= 0 && j < rows) atomicOr(&kept[j >> 5], 1u << (j & 31));
  }
  __syncthreads();
  for (int i = tid; i < kStatChunk; i += DM_THREADS) {
    const bool del = i < rows && !((kept[i >> 5] >> (i & 31)) & 1u);
    const float w = del ? sc[t0 + i] : 0.f;
    // w = w1 + w2 + w3 with every part a bf16 value (truncations: each takes the next eight significant bits)
    const uint32_t b1 = __float_as_uint(w) & 0xffff0000u;
    const float r1 = w - __uint_as_float(b1);
    const uint32_t b2 = __float_as_uint(r1) & 0xffff0000u;
    const float r2 = r1 - __uint_as_float(b2);
    wq[0][i] = (uint16_t)(b1 >> 16);
    wq[1][i] = (uint16_t)(b2 >> 16);
    wq[2][i] = (uint16_t)(__float_as_uint(r2) >> 16);
    wq[3][i] = del ? (uint16_t)0x3f80 : (uint16_t)0;
  }
  // (visible to everyone after the first barrier of the pipeline below)

  dm_f32x16 acc[DM_NACC];
#pragma unroll
  for (int t = 0; t < DM_NACC; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;

  // 16-byte pieces through registers (two per thread and tile), two tiles ahead of the products
  const int pc = lane & 15;
  uint4 pre[2][2];
  auto fetch = [&](uint4 (&dst)[2], int r0) {
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int r = min(r0 + gs_row<DM_WAVES>(wave, lane, q), rows - 1);      // clamped: rows past the end are zeroed in put
      dst[q] = *(const uint4*)(Vh + (size_t)(t0 + r) * DM_D + pc * 8);
    }
  };
  // retained rows and rows past the end are staged as zeros
  auto put = [&](const uint4 (&src)[2], int buf, int r0) {
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int rl = gs_row<DM_WAVES>(wave, lane, q);
      const int r = r0 + rl;
      const uint32_t kbit = (kept[(r >> 5) & (kStatChunk / 32 - 1)] >> (r & 31)) & 1u;
      gs_put(stage[buf], rl, lane, src[q], (r < rows) && !kbit);
    }
  };
  const int wj = wave & 3, wh = wave >> 2;
  const DmTiles tl3 = dm_wave_tiles(wj);
  const int oW = wj * 32, oA = tl3.a * 32, oB = tl3.b * 32, oC = tl3.c * 32;      // operand column blocks (words)
  auto compute = [&](const uint32_t* st, int r0) {
#pragma unroll 1
    for (int kk = 0; kk < 2; ++kk) {
      const int ks = 2 * wh + kk;
      DmFrag fW, f0, fA, fB, fC, e;
      gs_frag(fW, st, ks, lane, oW); gs_frag(f0, st, ks, lane, 0);
      gs_frag(fA, st, ks, lane, oA); gs_frag(fB, st, ks, lane, oB); gs_frag(fC, st, ks, lane, oC);
      // the sums' operand: row lr < 4 of it holds eight tokens' entries of weight part lr (or of the ones); the address is
      // clamped so that every lane loads, the other rows are cleared
      e.q = *(const uint4*)(&wq[lr & 3][r0 + ks * 16 + lh * 8]);
      if (lr >= 4) e.q = make_uint4(0u, 0u, 0u, 0u);
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fW.v, f0.v, acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fA.v, fB.v, acc[1], 0, 0, 0);
      acc[2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fC.v, fB.v, acc[2], 0, 0, 0);
      acc[3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(e.v, fW.v, acc[3], 0, 0, 0);
    }
  };
  fetch(pre[0], 0);
  fetch(pre[1], DM_TILE);
  __syncthreads();                       // wq and kept complete
  put(pre[0], 0, 0);
  fetch(pre[0], 2 * DM_TILE);
  lds_barrier();
#pragma unroll 1
  for (int r0 = 0; r0 < rows; r0 += 2 * DM_TILE) {
    // even tile: in stage[0]; pre[1] holds tile r0+64, pre[0] holds tile r0+128
    compute(stage[0], r0);
    put(pre[1], 1, r0 + DM_TILE);
    fetch(pre[1], r0 + 3 * DM_TILE);
    lds_barrier();                      // LDS only: the loads just issued stay in flight across the barrier
    if (r0 + DM_TILE < rows) compute(stage[1], r0 + DM_TILE);
    put(pre[0], 0, r0 + 2 * DM_TILE);
    fetch(pre[0], r0 + 4 * DM_TILE);
    lds_barrier();
  }

  // ---- the two halves' accumulators meet: waves 4 - 7 hand theirs over through LDS (the staging buffers are free after
  // the loop's last barrier), two products at a time; waves 0 - 3 add them to their own
  {
    float* xch = (float*)&stage[0][0];                 // [4 (j)][2][16][64] floats = 32 KB
#pragma unroll
    for (int round = 0; round < 2; ++round) {
      if (round) __syncthreads();
      if (wh == 1) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int i = 0; i < 16; ++i) xch[((wj * 2 + t) * 16 + i) * 64 + lane] = acc[round * 2 + t][i];
      }
      __syncthreads();
      if (wh == 0) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int i = 0; i < 16; ++i) acc[round * 2 + t][i] += xch[((wj * 2 + t) * 16 + i) * 64 + lane];
      }
    }
  }
  // ---- results (waves 0 - 3): the 32 x 32 tiles of the Gram matrix on and below the diagonal (row-major in the d x d
  // partial, so the stores are row segments; the tiles above the diagonal are left unwritten, the reader mirrors)
  float* out = gram_part + ((size_t)head * nstat + chunk) * gram_stride(DM_D);
  float tr = 0.f;                                      // this lane's share of the trace (the squared norms)
  if (wh == 0) {
    const int trb[3] = {wj, tl3.a, tl3.c}, tcb[3] = {0, tl3.b, tl3.b};
#pragma unroll
    for (int t = 0; t < 3; ++t) {
      if (t < 2 || tl3.third) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int rw = (i >> 2) * 8 + lh * 4 + (i & 3);
          out[(trb[t] * 32 + rw) * DM_D + tcb[t] * 32 + lr] = acc[t][i];
          if (trb[t] == tcb[t] && rw == lr) tr += acc[t][i];
        }
      }
    }
    // ---- weighted sum and plain sum: rows 0 - 3 of the sums tile
    if (lane < 32) {
      const int col = wj * 32 + lane;
      out[DM_D * DM_D + col] = (acc[3][0] + acc[3][1]) + acc[3][2];
      out[DM_D * DM_D + DM_D + col] = acc[3][3];
    }
  }
  for (int off = 32; off > 0; off >>= 1) tr += __shfl_xor(tr, off);
  if (lane == 0) red[wave] = tr;
  __syncthreads();
  if (tid == 0) out[DM_D * DM_D + 2 * DM_D] = (red[0] + red[1]) + (red[2] + red[3]);
}

// The active head whose number (in head order) is `target`, or -1; every thread gets it.  s_i has DM_WAVES + 1 entries.
__device__ int dm_active_head(const HeadState* __restrict__ state, int heads, int target, int* s_i) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (threadIdx.x == 0) s_i[DM_WAVES] = -1;
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
    if (p && before + __popcll(mask & ((1ull << lane) - 1ull)) == target) s_i[DM_WAVES] = h;
    base += tot;
    if (base > target) break;                        // uniform: found
  }
  __syncthreads();
  return s_i[DM_WAVES];
}

// grid (chunks, heads): workgroup (c, h) takes chunk c of head h.  With compact != 0 the grid is (chunks, a few rows) and
// row y takes the active heads number y, y + rows, ... (found by scanning the head states): for calls in which the
// certificate settles nearly every head, so that a launch over all heads would consist of workgroups that exit at once.
__global__ __launch_bounds__(DM_THREADS, 4) void k_bf_del_stats_mfma(const uint16_t* __restrict__ V,
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
  __shared__ int s_i[DM_WAVES + 1];
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
