// Attention-mass scores (Eq. 1) on the matrix cores: bf16 operands, fp32 accumulation
// (v_mfma_f32_32x32x16_bf16), head_dim 128.
//
// A column sum of softmax rows needs every row's normaliser before any column can be summed, so
// K is streamed twice: pass A gives each query row's (max, sum-exp) over each contiguous range of
// tokens a workgroup walks, pass B first folds the ranges of its head into the rows' log-sum-exp
// (in its prologue), then recomputes the logits and sums exp(logit - lse[row]) over the rows.  Both passes use the same register fragments of Q and K:
// an MFMA operand fragment holds, for lane l, 8 consecutive head_dim entries (l/32)*8.. of
// row l%32, for either operand, so swapping the two operands transposes the 32x32 output tile.
//   pass A computes (tokens x query rows): a lane then owns ONE query row per row block, and the
//          running (max, sum) needs two registers per row block;
//   pass B computes (query rows x tokens): a lane owns ONE token, and the column sum is an
//          in-lane sum plus one cross-lane add.
// The whole Q operand of a 128-row group lives in registers for the lifetime of a workgroup;
// K fragments are loaded straight from global memory in 16-byte pieces, one tile ahead.
#include "common.hpp"

namespace obf {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int SM_THREADS = 256;
constexpr int SM_WAVES = 4;
// The kernels are instantiated for (RB, KBUF) = (4, 3) and (5, 2): RB 32-row blocks of query rows per workgroup (RB * 32 = 128
// or 160 rows, their Q operand in RB * 32 registers per lane) and KBUF rotating K fragment buffers.  RB * KBUF is even, so the
// two accumulators keep alternating across the iterations of the tile loop.
constexpr int SM_D = 128;
constexpr int SM_KK = SM_D / 16;         // MFMA k-steps
constexpr int SM_TILE = 32;              // tokens per MFMA tile
constexpr float kLog2e = 1.4426950408889634f;
constexpr int kScoreOneLaunchTokens = 768;   // prompts up to this length take both score passes in one launch (a tie with two launches near 1024)

union Frag { uint4 u; bf16x8 v; };

// Rows past R and tokens past t_end are clamped to the last valid one instead of being predicated: their
// results are never used (padded rows get lse = +inf in pass B and are not written in pass A; tokens past the
// end are masked by index), and branch-free loads keep the fragments in registers.
template <int RB>
__device__ __forceinline__ void load_q(Frag (&qf)[RB][SM_KK], const uint16_t* __restrict__ Qh, int row0, int R, int lane) {
  const int r = lane & 31, kh = (lane >> 5) * 8;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int row = min(row0 + rb * 32 + r, R - 1);
    const uint4* p = (const uint4*)(Qh + (size_t)row * SM_D + kh);
#pragma unroll
    for (int kk = 0; kk < SM_KK; ++kk) qf[rb][kk].u = p[kk * 2];
  }
}

__device__ __forceinline__ void load_k(Frag (&kf)[SM_KK], const uint16_t* __restrict__ Kh, int tok0, int t_end, int lane) {
  const int t = min(tok0 + (lane & 31), t_end - 1), kh = (lane >> 5) * 8;
  const uint4* p = (const uint4*)(Kh + (size_t)t * SM_D + kh);
#pragma unroll
  for (int kk = 0; kk < SM_KK; ++kk) kf[kk].u = p[kk * 2];
}

// ------------------------------------------------------------------------------------------------
// Shared tile machinery.  A wave walks the 32-token tiles wave, wave+4, ... of its chunk.  The MFMAs of
// tile i+1 are issued in the same basic block as the vector-ALU epilogue of tile i (two accumulator
// sets, two K fragment buffers), so that the matrix pipe and the vector ALU overlap within the one
// wave a SIMD holds.

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }   // v_exp_f32, denormal results flush to 0

// MFMA chain of one 32-row block against one 32-token tile (8 k-steps of 16).
template <bool TOKENS_BY_ROWS>
__device__ __forceinline__ void block_mfma(f32x16& acc, const Frag (&kf)[SM_KK], const Frag (&qf)[SM_KK]) {
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
  for (int kk = 0; kk < SM_KK; ++kk) {
    if (TOKENS_BY_ROWS) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk].v, qf[kk].v, acc, 0, 0, 0);
    else acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[kk].v, kf[kk].v, acc, 0, 0, 0);
  }
}

// Pass A epilogue of one row block of a tile whose 32 tokens are all valid.  acc[i] is the raw dot product
// of token tok + (i/4)*8 + (lane/32)*4 + (i%4) with query row row0 + rb*32 + lane%32.  m is the running
// maximum in raw units, l the running sum of exp2((raw - m) a2) in double.
template <int NRB>
struct StatsEp {
  float (&m)[NRB];
  double (&l)[NRB];
  float a2;
  template <int RB>
  __device__ __forceinline__ void block(const f32x16& acc, int) {
    float mx = fmaxf(fmaxf(acc[0], acc[1]), acc[2]);
#pragma unroll
    for (int i = 3; i < 15; i += 2) mx = fmaxf(fmaxf(mx, acc[i]), acc[i + 1]);
    mx = fmaxf(mx, acc[15]);
    const float mo = m[RB];
    const float mn = fmaxf(mo, mx);
    const float off = mn * a2;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
    for (int i = 0; i < 16; i += 4) {
      s0 += fast_exp2(fmaf(acc[i], a2, -off));
      s1 += fast_exp2(fmaf(acc[i + 1], a2, -off));
      s2 += fast_exp2(fmaf(acc[i + 2], a2, -off));
      s3 += fast_exp2(fmaf(acc[i + 3], a2, -off));
    }
    const float ts = (s0 + s1) + (s2 + s3);
    const float sc = fast_exp2((mo - mn) * a2);          // 0 on the first tile (mo = -inf), 1 when the maximum stands
    l[RB] = fma(l[RB], (double)sc, (double)ts);
    m[RB] = mn;
    // Pin the update here: its results are only read by the next tile, so the optimiser would otherwise sink all
    // epilogues of a loop iteration behind the matrix instructions, and the two pipes would take turns instead of
    // running side by side.
    asm volatile("" : "+v"(l[RB]), "+v"(m[RB]));
  }
};

// Same for a ragged tile: tokens at or past t_end are left out.
__device__ __forceinline__ void stats_block_ragged(const f32x16& acc, float& m, double& l, float a2, int tok, int t_end,
                                                   int lane) {
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int t = tok + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
    if (t < t_end) mx = fmaxf(mx, acc[i]);
  }
  const float mo = m;
  const float mn = fmaxf(mo, mx);
  if (mn > -INFINITY) {
    const float off = mn * a2;
    float ts = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int t = tok + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
      if (t < t_end) ts += fast_exp2(fmaf(acc[i], a2, -off));
    }
    const float sc = (mo > -INFINITY) ? fast_exp2((mo - mn) * a2) : 0.f;
    l = fma(l, (double)sc, (double)ts);
    m = mn;
  }
}

// Pass B epilogue: acc[i] is the raw dot product of query row row0 + rb*32 + (i/4)*8 + (lane/32)*4 + (i%4) with
// token tok + lane%32; b2 holds lse[row] * log2(e) for the same (rb, i).  The column sum of a tile is
// complete after its last row block.
template <int NRB>
struct MassEp {
  const float (&b2)[NRB][16];
  float a2;
  float* __restrict__ dst;
  int t_end, lane;
  float c0, c1, c2, c3;
  template <int RB>
  __device__ __forceinline__ void block(const f32x16& acc, int tok) {
    if (RB == 0) { c0 = 0.f; c1 = 0.f; c2 = 0.f; c3 = 0.f; }
#pragma unroll
    for (int i = 0; i < 16; i += 4) {
      c0 += fast_exp2(fmaf(acc[i], a2, -b2[RB][i]));
      c1 += fast_exp2(fmaf(acc[i + 1], a2, -b2[RB][i + 1]));
      c2 += fast_exp2(fmaf(acc[i + 2], a2, -b2[RB][i + 2]));
      c3 += fast_exp2(fmaf(acc[i + 3], a2, -b2[RB][i + 3]));
    }
    if (RB == NRB - 1) {
      float col = (c0 + c1) + (c2 + c3);
      const float other = __shfl_xor(col, 32);
      col = (lane < 32) ? (col + other) : (other + col);
      const int t = tok + (lane & 31);
      if (lane < 32 && t < t_end) dst[t] = col;
    }
  }
};

// Software pipeline over the tiles first, first + STEP, ... of one wave, at row-block granularity: micro-stage
// (tile t, row block rb) issues the MFMA chain of the NEXT (tile, row block) and, in the same basic block,
// runs the vector-ALU epilogue of the current one, so the matrix pipe and the vector ALU overlap within the
// one wave a SIMD holds.  Two 16-register accumulators alternate; three K fragment buffers rotate, and the load
// of tile t+3 is issued once the last chain of tile t has been issued (almost three tiles of work ahead of
// its first use: the memory latency is covered by two tiles' worth of compute).
template <bool TOKENS_BY_ROWS, int RB, int KBUF, int U, class Ep>
__device__ __forceinline__ void micro_stage(const uint16_t* __restrict__ Kh, int first, int step, int n, int t_end, int lane, int i,
                                            const Frag (&qf)[RB][SM_KK], Frag (&kb)[KBUF][SM_KK], f32x16 (&acc)[2], Ep& ep,
                                            bool guarded) {
  constexpr int rb = U % RB, tl = U / RB;                 // current row block, tile offset within the group of KBUF
  constexpr int rbn = (U + 1) % RB, tln = (U + 1) / RB;   // next
  const int tile = i + tl, tilen = i + tln;
  if (guarded && tile >= n) return;
  if (!guarded || tilen < n) block_mfma<TOKENS_BY_ROWS>(acc[(U + 1) & 1], kb[tln % KBUF], qf[rbn]);
  ep.template block<rb>(acc[U & 1], first + tile * step);
  if (rb == RB - 1 && tile + KBUF < n) load_k(kb[tl % KBUF], Kh, first + (tile + KBUF) * step, t_end, lane);
  __builtin_amdgcn_sched_barrier(0);      // keep the scheduler from merging micro-stages (register pressure)
}

// The RB * KBUF micro-stages of one iteration of the tile loop, in order.
template <bool TOKENS_BY_ROWS, int RB, int KBUF, int U, class Ep>
__device__ __forceinline__ void stage_sequence(const uint16_t* __restrict__ Kh, int first, int step, int n, int t_end, int lane,
                                               int i, const Frag (&qf)[RB][SM_KK], Frag (&kb)[KBUF][SM_KK], f32x16 (&acc)[2],
                                               Ep& ep, bool guarded) {
  if constexpr (U < RB * KBUF) {
    micro_stage<TOKENS_BY_ROWS, RB, KBUF, U>(Kh, first, step, n, t_end, lane, i, qf, kb, acc, ep, guarded);
    stage_sequence<TOKENS_BY_ROWS, RB, KBUF, U + 1>(Kh, first, step, n, t_end, lane, i, qf, kb, acc, ep, guarded);
  }
}

template <bool TOKENS_BY_ROWS, int RB, int KBUF, class Ep>
__device__ __forceinline__ void run_tiles(const uint16_t* __restrict__ Kh, int first, int step, int n, int t_end, int lane,
                                          const Frag (&qf)[RB][SM_KK], Ep& ep) {
  static_assert((RB * KBUF) % 2 == 0, "the accumulators alternate per micro-stage");
  if (n <= 0) return;
  Frag kb[KBUF][SM_KK];
  f32x16 acc[2];
#pragma unroll
  for (int t = 0; t < KBUF; ++t)
    if (t < n) load_k(kb[t], Kh, first + t * step, t_end, lane);
  block_mfma<TOKENS_BY_ROWS>(acc[0], kb[0], qf[0]);
  int i = 0;
  for (; i + KBUF < n; i += KBUF)                       // KBUF whole tiles and the first chain of the next exist
    stage_sequence<TOKENS_BY_ROWS, RB, KBUF, 0>(Kh, first, step, n, t_end, lane, i, qf, kb, acc, ep, false);
  stage_sequence<TOKENS_BY_ROWS, RB, KBUF, 0>(Kh, first, step, n, t_end, lane, i, qf, kb, acc, ep, true);
}

// Static partition of the flattened (head, tile) space over the persistent workgroups.
struct Part {
  int TH;        // 32-token tiles per head
  int T;         // tiles per workgroup range
  long TT;       // heads * TH
  long kstride;  // elements between consecutive heads of K
};

// ------------------------------------------------------------------------------------------------
// Pass A.  grid = G ranges x RG row groups, one workgroup per compute unit; a workgroup walks its range of
// tiles segment by segment (a segment = the part of one head inside the range) and leaves one partial
// (max, sum-exp) per query row and segment.
template <int RB, int KBUF>
__global__ __launch_bounds__(SM_THREADS, 1) void k_score_stats_mfma(const uint16_t* __restrict__ K,
                                                                    const uint16_t* __restrict__ Q,
                                                                    double* __restrict__ stats_part, int N, int R,
                                                                    int RG, Part pt, int nslot) {
  __shared__ double s_m[SM_WAVES][(RB * 32)], s_l[SM_WAVES][(RB * 32)];
  // Workgroups are dealt to the 8 XCDs round-robin.  The RG workgroups that stream the same K range (one per row
  // group) get block indices 8 apart, so they run on one XCD side by side and share its L2.
  const int blk_group = blockIdx.x / (8 * RG), blk_in = blockIdx.x - blk_group * (8 * RG);
  const int range = blk_group * 8 + (blk_in & 7), rg = blk_in >> 3;
  if ((long)range * pt.T >= pt.TT) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row0 = rg * (RB * 32);
  const float a2 = kLog2e / sqrtf((float)SM_D);
  constexpr int STEP = SM_WAVES * SM_TILE;
  const long gs = (long)range * pt.T;
  const long ge = min(pt.TT, gs + pt.T);

  for (long cur = gs; cur < ge;) {
    const int head = (int)(cur / pt.TH);
    const long hs = (long)head * pt.TH;
    const long se = min(ge, hs + pt.TH);
    const int ta = (int)(cur - hs) * SM_TILE, tb = min(N, (int)(se - hs) * SM_TILE);
    const int slot = range - (int)(hs / pt.T);
    const uint16_t* Kh = K + (size_t)head * pt.kstride;
    const uint16_t* Qh = Q + (size_t)head * R * SM_D;

    Frag qf[RB][SM_KK];
    load_q(qf, Qh, row0, R, lane);
    float m[RB];
    double l[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) { m[rb] = -INFINITY; l[rb] = 0.0; }
    const int first = ta + wave * SM_TILE;
    const int nfull = (tb - first >= SM_TILE) ? ((tb - first - SM_TILE) / STEP + 1) : 0;
    StatsEp<RB> ep{m, l, a2};
    run_tiles<true, RB, KBUF>(Kh, first, STEP, nfull, tb, lane, qf, ep);
    {
      const int tok = first + nfull * STEP;          // a ragged last tile, if any
      if (tok < tb) {
        Frag kr[SM_KK];
        load_k(kr, Kh, tok, tb, lane);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
          f32x16 accr;
          block_mfma<true>(accr, kr, qf[rb]);
          stats_block_ragged(accr, m[rb], l[rb], a2, tok, tb, lane);
        }
      }
    }
    // fold the two lane halves (same query row, different tokens), then the four waves
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const float mo = __shfl_xor(m[rb], 32);
      const double lo = __shfl_xor(l[rb], 32);
      const float mn = fmaxf(m[rb], mo);
      double a = 0.0, b = 0.0;
      // (the exponents are differences of two float maxima: a single-precision exp2 loses nothing they still carry)
      if (m[rb] > -INFINITY) a = l[rb] * (double)fast_exp2((m[rb] - mn) * a2);
      if (mo > -INFINITY) b = lo * (double)fast_exp2((mo - mn) * a2);
      if (lane < 32) { s_m[wave][rb * 32 + lane] = (double)mn * (double)a2; s_l[wave][rb * 32 + lane] = a + b; }
    }
    __syncthreads();
    if (threadIdx.x < (RB * 32)) {
      const int row = row0 + threadIdx.x;
      if (row < R) {
        double M = -INFINITY;
        for (int w = 0; w < SM_WAVES; ++w) M = fmax(M, s_m[w][threadIdx.x]);
        double L = 0.0;
        for (int w = 0; w < SM_WAVES; ++w)
          if (s_m[w][threadIdx.x] > -INFINITY) L += s_l[w][threadIdx.x] * exp2(s_m[w][threadIdx.x] - M);
        double* o = stats_part + (((size_t)head * nslot + slot) * R + row) * 2;
        o[0] = M * 0.6931471805599453;     // log2 units -> natural log
        o[1] = L;
      }
    }
    __syncthreads();
    cur = se;
  }
}

// ------------------------------------------------------------------------------------------------
// Pass B.  Same partition.  First folds the head's partials into log-sum-exp (every workgroup that touches
// a head computes the same values; the one holding the head's first tile also writes row_lse), then
// out = scores (RG == 1) or the row group's partial column sums.
template <int RB, int KBUF>
__global__ __launch_bounds__(SM_THREADS, 1) void k_score_mass_mfma(const uint16_t* __restrict__ K,
                                                                   const uint16_t* __restrict__ Q,
                                                                   const double* __restrict__ stats_part,
                                                                   double* __restrict__ row_lse,
                                                                   float* __restrict__ out, int N, int R, int RG,
                                                                   size_t rg_stride, Part pt, int nslot) {
  __shared__ double s_lse[(RB * 32)];
  // Workgroups are dealt to the 8 XCDs round-robin.  The RG workgroups that stream the same K range (one per row
  // group) get block indices 8 apart, so they run on one XCD side by side and share its L2.
  const int blk_group = blockIdx.x / (8 * RG), blk_in = blockIdx.x - blk_group * (8 * RG);
  const int range = blk_group * 8 + (blk_in & 7), rg = blk_in >> 3;
  if ((long)range * pt.T >= pt.TT) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row0 = rg * (RB * 32);
  const float a2 = kLog2e / sqrtf((float)SM_D);
  constexpr int STEP = SM_WAVES * SM_TILE;
  const long gs = (long)range * pt.T;
  const long ge = min(pt.TT, gs + pt.T);

  // The range is walked BACKWARDS (last segment first, last tile first): the first pass has just streamed it
  // forwards, so its end is what the memory-side cache still holds.
  for (long se = ge; se > gs;) {
    const int head = (int)((se - 1) / pt.TH);
    const long hs = (long)head * pt.TH;
    const long cur = max(gs, hs);
    const int ta = (int)(cur - hs) * SM_TILE, tb = min(N, (int)(se - hs) * SM_TILE);
    const uint16_t* Kh = K + (size_t)head * pt.kstride;
    const uint16_t* Qh = Q + (size_t)head * R * SM_D;
    float* dst = out + (size_t)rg * rg_stride + (size_t)head * N;

    __syncthreads();
    if (threadIdx.x < (RB * 32)) {
      const int row = row0 + threadIdx.x;
      double lse = INFINITY;                                   // padded rows: exp2(-inf) = 0
      if (row < R) {
        const int s_first = (int)(hs / pt.T), s_last = (int)((hs + pt.TH - 1) / pt.T);
        const double* p = stats_part + ((size_t)head * nslot * R + row) * 2;
        double M = -INFINITY;
        for (int sl = 0; sl <= s_last - s_first; ++sl) M = fmax(M, p[(size_t)sl * R * 2]);
        double L = 0.0;
        for (int sl = 0; sl <= s_last - s_first; ++sl) {
          const double pm = p[(size_t)sl * R * 2], pl = p[(size_t)sl * R * 2 + 1];
          if (pm != -INFINITY) L += pl * exp(pm - M);
        }
        lse = M + log(L);
        if (cur == hs) row_lse[(size_t)head * R + row] = lse;
      }
      s_lse[threadIdx.x] = lse;
    }
    __syncthreads();

    Frag qf[RB][SM_KK];
    load_q(qf, Qh, row0, R, lane);
    float b2[RB][16];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int i = 0; i < 16; ++i)
        b2[rb][i] = (float)(s_lse[rb * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3)] * 1.4426950408889634);

    const int first = ta + wave * SM_TILE;
    const int nt = (first < tb) ? ((tb - first - 1) / STEP + 1) : 0;      // tiles of this wave, the last may be ragged
    MassEp<RB> ep{b2, a2, dst, tb, lane, 0.f, 0.f, 0.f, 0.f};
    run_tiles<false, RB, KBUF>(Kh, first + (nt - 1) * STEP, -STEP, nt, tb, lane, qf, ep);
    se = cur;
  }
}

// ------------------------------------------------------------------------------------------------
// Both passes in one launch, for short prompts (a head's tiles are few and one row group covers the query rows): one
// workgroup per head keeps Q in registers, takes the row maxima and sums over the head's tokens, forms the row
// log-sum-exp in LDS and walks the same tokens again, backwards, for the masses.  Same arithmetic, in the same order, as
// the two launches make of a head that lies inside one range.
template <int RB, int KBUF>
__global__ __launch_bounds__(SM_THREADS, 1) void k_score_head_mfma(const uint16_t* __restrict__ K,
                                                                   const uint16_t* __restrict__ Q,
                                                                   double* __restrict__ row_lse, float* __restrict__ out,
                                                                   int N, int R, long kstride) {
  __shared__ double s_m[SM_WAVES][(RB * 32)], s_l[SM_WAVES][(RB * 32)];
  __shared__ double s_lse[(RB * 32)];
  const int head = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float a2 = kLog2e / sqrtf((float)SM_D);
  constexpr int STEP = SM_WAVES * SM_TILE;
  const uint16_t* Kh = K + (size_t)head * kstride;
  const uint16_t* Qh = Q + (size_t)head * R * SM_D;
  float* dst = out + (size_t)head * N;
  const int first = wave * SM_TILE;

  Frag qf[RB][SM_KK];
  load_q(qf, Qh, 0, R, lane);
  {
    float m[RB];
    double l[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) { m[rb] = -INFINITY; l[rb] = 0.0; }
    const int nfull = (N - first >= SM_TILE) ? ((N - first - SM_TILE) / STEP + 1) : 0;
    StatsEp<RB> ep{m, l, a2};
    run_tiles<true, RB, KBUF>(Kh, first, STEP, nfull, N, lane, qf, ep);
    {
      const int tok = first + nfull * STEP;          // a ragged last tile, if any
      if (tok < N) {
        Frag kr[SM_KK];
        load_k(kr, Kh, tok, N, lane);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
          f32x16 accr;
          block_mfma<true>(accr, kr, qf[rb]);
          stats_block_ragged(accr, m[rb], l[rb], a2, tok, N, lane);
        }
      }
    }
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {                // the two lane halves, then (below) the four waves
      const float mo = __shfl_xor(m[rb], 32);
      const double lo = __shfl_xor(l[rb], 32);
      const float mn = fmaxf(m[rb], mo);
      double a = 0.0, b = 0.0;
      if (m[rb] > -INFINITY) a = l[rb] * (double)fast_exp2((m[rb] - mn) * a2);
      if (mo > -INFINITY) b = lo * (double)fast_exp2((mo - mn) * a2);
      if (lane < 32) { s_m[wave][rb * 32 + lane] = (double)mn * (double)a2; s_l[wave][rb * 32 + lane] = a + b; }
    }
  }
  __syncthreads();
  if (threadIdx.x < (RB * 32)) {
    const int row = threadIdx.x;
    double lse = INFINITY;                                     // padded rows: exp2(-inf) = 0
    if (row < R) {
      double M = -INFINITY;
      for (int w = 0; w < SM_WAVES; ++w) M = fmax(M, s_m[w][row]);
      double L = 0.0;
      for (int w = 0; w < SM_WAVES; ++w)
        if (s_m[w][row] > -INFINITY) L += s_l[w][row] * exp2(s_m[w][row] - M);
      lse = M * 0.6931471805599453 + log(L);                   // log2 units -> natural log
      row_lse[(size_t)head * R + row] = lse;
    }
    s_lse[row] = lse;
  }
  __syncthreads();
  float b2[RB][16];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int i = 0; i < 16; ++i)
      b2[rb][i] = (float)(s_lse[rb * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3)] * 1.4426950408889634);
  const int nt = (first < N) ? ((N - first - 1) / STEP + 1) : 0;          // tiles of this wave, the last may be ragged
  MassEp<RB> ep{b2, a2, dst, N, lane, 0.f, 0.f, 0.f, 0.f};
  run_tiles<false, RB, KBUF>(Kh, first + (nt - 1) * STEP, -STEP, nt, N, lane, qf, ep);
}

// scores = sum of the row groups' partial column sums (fixed order)
__global__ void k_score_sum_groups(const float* __restrict__ part, float* __restrict__ scores, size_t n, int RG,
                                   size_t rg_stride) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float s = 0.f;
  for (int g = 0; g < RG; ++g) s += part[(size_t)g * rg_stride + i];
  scores[i] = s;
}

bool mfma_score_supported(const Dims& m) {
  return m.dtype == OBF_BF16 && m.d == SM_D;
}

obf_status_t launch_score_mfma(const Dims& m, const Workspace& w, char* ws, const void* K, const void* Q,
                               float* scores, double* row_lse, hipStream_t st) {
  double* stats_part = (double*)(ws + w.stats_part);
  const int RG = w.rgroups;
  const size_t rg_stride = (size_t)m.heads * m.N;
  float* part = (RG > 1) ? (float*)(ws + w.score_part) : scores;
  Part pt;
  pt.TH = w.tiles_per_head; pt.T = w.tiles_per_range; pt.TT = (long)m.heads * w.tiles_per_head;
  pt.kstride = (long)m.kvs * SM_D;
  dim3 grid(((w.nranges + 7) / 8) * 8 * RG);
  const bool five = score_rows_per_group(m.R) == 160;     // five row blocks per workgroup, two K buffers (e.g. 320 rows = 2 x 160)
  if (RG == 1 && !five && m.N <= kScoreOneLaunchTokens) {  // short prompts: both passes in one launch, a workgroup per head
    ProfScope prof_(ST_SCORE_STATS, st);
    hipLaunchKernelGGL((k_score_head_mfma<4, 3>), dim3(m.heads), dim3(SM_THREADS), 0, st, (const uint16_t*)K, (const uint16_t*)Q,
                       row_lse, scores, m.N, m.R, pt.kstride);
    return check_launch("score, one launch per call (mfma)");
  }
  { ProfScope prof_(ST_SCORE_STATS, st);
    if (five)
      hipLaunchKernelGGL((k_score_stats_mfma<5, 2>), grid, dim3(SM_THREADS), 0, st, (const uint16_t*)K, (const uint16_t*)Q,
                         stats_part, m.N, m.R, RG, pt, w.nslot);
    else
      hipLaunchKernelGGL((k_score_stats_mfma<4, 3>), grid, dim3(SM_THREADS), 0, st, (const uint16_t*)K, (const uint16_t*)Q,
                         stats_part, m.N, m.R, RG, pt, w.nslot); }
  if (check_launch("score stats (mfma)") != OBF_OK) return OBF_ERR_HIP;
  { ProfScope prof_(ST_SCORE_MASS, st);
    if (five)
      hipLaunchKernelGGL((k_score_mass_mfma<5, 2>), grid, dim3(SM_THREADS), 0, st, (const uint16_t*)K, (const uint16_t*)Q,
                         (const double*)stats_part, row_lse, part, m.N, m.R, RG, rg_stride, pt, w.nslot);
    else
      hipLaunchKernelGGL((k_score_mass_mfma<4, 3>), grid, dim3(SM_THREADS), 0, st, (const uint16_t*)K, (const uint16_t*)Q,
                         (const double*)stats_part, row_lse, part, m.N, m.R, RG, rg_stride, pt, w.nslot); }
  if (check_launch("score mass (mfma)") != OBF_OK) return OBF_ERR_HIP;
  if (RG > 1) {
    const size_t n = (size_t)m.heads * m.N;
    hipLaunchKernelGGL(k_score_sum_groups, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, part, scores, n, RG,
                       rg_stride);
    if (check_launch("score sum groups") != OBF_OK) return OBF_ERR_HIP;
  }
  return OBF_OK;
}

}  // namespace obf
