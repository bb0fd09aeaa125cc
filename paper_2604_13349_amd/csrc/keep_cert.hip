// Fast decision "the retained values span all of R^d" (then Eq. 3's residual is identically zero and
// the head stays plain eviction) for bf16 caches with head_dim 128 and more retained rows than
// head_dim.  It is a sufficient test only: heads it cannot certify go to the reference-precision
// basis kernel.
//
//   G   = V_s^T V_s over a strided subset V_s of the retained rows (all rows up to 512), on the matrix
//         cores: products of bf16 values are exact in fp32, accumulation is fp32;
//   mu  = (max(n, d) 2^-23)^2 ||V_keep||_F^2;
//   S   = D^-1/2 G D^-1/2 with D = diag(G): G - mu I is positive definite iff S - mu D^-1 is;
//   if the LDL^T factorisation of S - mu D^-1 - eps I (eps: allowance for the fp32 error of G and of the
//   factorisation, relative to trace(S) = d) runs through with positive pivots, then
//   sigma_min(V_keep)^2 >= lambda_min(G) > (max(n, d) 2^-23)^2 sigma_max(V_keep)^2, i.e. every singular
//   value is above the rank rule's threshold: r = d.
#include "common.hpp"
#include "gram_stage.hpp"
#include "wave_ops.hpp"

namespace obf {

typedef gs_f32x16 f32x16;

constexpr int KC_THREADS = 256;
constexpr int KC_WAVES = KC_THREADS / 64;
constexpr int KC_D = GS_D;
constexpr int KC_TILE = GS_TILE;         // rows staged per iteration
constexpr int KC_MINROWS = 512;          // rows entering G: all up to 512, else about max(512, n/4) at a constant stride
constexpr float kCertErr = 1.6e-5f;      // allowance for fp32 Gram + factorisation error, relative to the trace of the scaled Gram matrix (= d)


// The lower triangle of G is ten 32x32 tiles (row block rb >= column block cb).  Each tile lives in one wave's
// registers from the Gram phase to the end of the factorisation: entry i of lane l is
// G[rb*32 + (i/4)*8 + (l/32)*4 + (i%4)][cb*32 + l%32].  No wave holds two tiles of the same column block, so the
// part of a step that the next pivot column waits for is at most one tile update per wave.
__device__ __forceinline__ void wave_tiles(int wave, int (&rb)[3], int (&cb)[3], int& nt) {
  if (wave == 0) { rb[0] = 0; cb[0] = 0; rb[1] = 1; cb[1] = 1; rb[2] = 3; cb[2] = 2; nt = 3; }
  else if (wave == 1) { rb[0] = 1; cb[0] = 0; rb[1] = 2; cb[1] = 1; rb[2] = 3; cb[2] = 3; nt = 3; }
  else if (wave == 2) { rb[0] = 2; cb[0] = 0; rb[1] = 3; cb[1] = 1; rb[2] = 0; cb[2] = 0; nt = 2; }
  else { rb[0] = 3; cb[0] = 0; rb[1] = 2; cb[1] = 2; rb[2] = 0; cb[2] = 0; nt = 2; }
}

template <bool via_idx>
__global__ __launch_bounds__(KC_THREADS, 2) void k_bf_keep_cert(const uint16_t* __restrict__ Vsrc /*via_idx ? V [heads][N][d] : gathered rows [heads][max_budget][d]*/,
                                                             const float* __restrict__ scores,
                                                             const int32_t* __restrict__ idx,
                                                             const int32_t* __restrict__ n_keep, int N, int max_budget,
                                                             int rank, HeadState* __restrict__ state,
                                                             int32_t* __restrict__ decided,
                                                             const double* __restrict__ fro_part /*optional: sums of squares of the retained rows, per gather block*/,
                                                             int fro_blocks, int scs, int kvs,
                                                             int want_sums /*0: the demand sums of a certified head (diagnostics only) are left at zero*/) {
  __shared__ __attribute__((aligned(16))) uint32_t stage[2][GS_STAGE_WORDS];
  __shared__ __attribute__((aligned(16))) float panel[2][KC_D][4];
  __shared__ float4 ypan[KC_D], lpan[KC_D];
  __shared__ __attribute__((aligned(16))) float isd[KC_D];
  __shared__ int s_bad;
  __shared__ double red[KC_THREADS / 64], red2[KC_THREADS / 64];
  const int head = blockIdx.x;
  const int n = n_keep[head];
  const int n_del = N - n;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform, kept in a scalar register
  const int lr = lane & 31, lh = lane >> 5;
  if (tid == 0) decided[head] = 0;
  if (!(rank > 0 && n > KC_D && n_del > 0)) return;
  const float* sc = scores + (size_t)head * scs;
  const int32_t* id = idx + (size_t)head * max_budget;
  const uint16_t* Vh = Vsrc + (size_t)head * (via_idx ? kvs : max_budget) * KC_D;
  auto row_of = [&](int r) -> size_t { return via_idx ? (size_t)id[r] : (size_t)r; };    // retained row r of the head
  const int cap = max(KC_MINROWS, n >> 2);
  const int stride = (n + cap - 1) / cap;
  const int rows = (n + stride - 1) / stride;
  int trb[3], tcb[3], nt;
  wave_tiles(wave, trb, tcb, nt);

  f32x16 acc[3];
#pragma unroll
  for (int t = 0; t < 3; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;

  // ---- Gram phase: rows staged 64 at a time through LDS (double buffered); the loads run two tiles ahead in
  // registers so that their latency is covered by the products of two tiles.  All waves run one instruction stream:
  // the operands of a wave's tiles are picked by LDS address (a wave with two tiles repeats its second product into an
  // accumulator nobody reads).
  const int pc = lane & 15;
  uint4 pre[2][4];
  auto fetch = [&](uint4 (&dst)[4], int r0) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int r = min(r0 + gs_row<KC_WAVES>(wave, lane, q), rows - 1);      // clamped: rows past the end are zeroed in put
      dst[q] = *(const uint4*)(Vh + row_of(r * stride) * KC_D + pc * 8);
    }
  };
  auto put = [&](const uint4 (&src)[4], int buf, int r0) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int rl = gs_row<KC_WAVES>(wave, lane, q);
      gs_put(stage[buf], rl, lane, src[q], r0 + rl < rows);
    }
  };
  const int oA0 = trb[0] * 32, oB0 = tcb[0] * 32, oA1 = trb[1] * 32, oB1 = tcb[1] * 32;
  const int oA2 = (nt > 2 ? trb[2] : trb[1]) * 32, oB2 = (nt > 2 ? tcb[2] : tcb[1]) * 32;
  auto compute = [&](const uint32_t* st) {
#pragma unroll
    for (int ks = 0; ks < KC_TILE / 16; ++ks) {
      GsFrag a0, b0, a1, b1, a2, b2;
      gs_frag(a0, st, ks, lane, oA0); gs_frag(b0, st, ks, lane, oB0);
      gs_frag(a1, st, ks, lane, oA1); gs_frag(b1, st, ks, lane, oB1);
      gs_frag(a2, st, ks, lane, oA2); gs_frag(b2, st, ks, lane, oB2);
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0.v, b0.v, acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1.v, b1.v, acc[1], 0, 0, 0);
      acc[2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2.v, b2.v, acc[2], 0, 0, 0);
    }
  };
  // The demand sums of Eq. 6 (diagnostics of a certified head) need sum(scores[idx]) and sum(scores): their first
  // batch of loads is issued here and consumed after the factorisation, so that its latency is hidden.
  int ej[8];
  const bool vec_scores = (N & 3) == 0 && ((uintptr_t)sc & 15) == 0;
  const int ns = want_sums ? n : 0, Ns = want_sums ? N : 0;          // extents of the two sums
#pragma unroll
  for (int u = 0; u < 8; ++u) { const int i = tid + u * KC_THREADS; ej[u] = (i < ns) ? id[i] : -1; }
  // tile j is staged in stage[j % 2]; the loads run two tiles ahead in registers
  fetch(pre[0], 0);
  fetch(pre[1], KC_TILE);
  put(pre[0], 0, 0);
  fetch(pre[0], 2 * KC_TILE);
  lds_barrier();
#pragma unroll 1
  for (int r0 = 0; r0 < rows; r0 += 2 * KC_TILE) {
    // even tile: in stage[0]; pre[1] holds tile r0+64, pre[0] holds tile r0+128
    compute(stage[0]);
    put(pre[1], 1, r0 + KC_TILE);
    fetch(pre[1], r0 + 3 * KC_TILE);
    lds_barrier();                      // LDS only: the loads just issued stay in flight across the barrier
    if (r0 + KC_TILE < rows) compute(stage[1]);
    put(pre[0], 0, r0 + 2 * KC_TILE);
    fetch(pre[0], r0 + 4 * KC_TILE);
    lds_barrier();
  }
  float ev[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) ev[u] = (ej[u] >= 0) ? sc[ej[u]] : 0.f;
  // ---- trace(G), ||V_keep||_F^2, shift
  // a lane holds a diagonal entry of a diagonal tile iff (lr % 8) / 4 == lh, at i = (lr / 8) * 4 + lr % 4
  const bool has_diag = ((lr & 7) >> 2) == lh;
  const int di = (lr >> 3) * 4 + (lr & 3);
  double part = 0.0;
#pragma unroll
  for (int t = 0; t < 3; ++t) {
    if (t < nt && trb[t] == tcb[t] && has_diag) {
      float v = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) if (i == di) v = acc[t][i];
      part += (double)v;
    }
  }
  for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off);
  if (lane == 0) red[wave] = part;
  __syncthreads();
  const double tr = (red[0] + red[1]) + (red[2] + red[3]);
  __syncthreads();
  double f2 = tr;
  if (stride > 1 && fro_part) {
    double p2 = 0.0;
    for (int b = tid; b < fro_blocks; b += KC_THREADS) p2 += fro_part[(size_t)head * fro_blocks + b];
    for (int off = 32; off > 0; off >>= 1) p2 += __shfl_xor(p2, off);
    if (lane == 0) red[wave] = p2;
    __syncthreads();
    f2 = (red[0] + red[1]) + (red[2] + red[3]);
    __syncthreads();
  } else if (stride > 1) {
    double p2 = 0.0;
    const int sub = tid >> 4, piece = tid & 15;
    for (int r0 = sub; r0 < n; r0 += 8 * (KC_THREADS / 16)) {          // 8 independent row pieces in flight per lane
      uint4 q[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int r = r0 + u * (KC_THREADS / 16);
        q[u] = (r < n) ? *(const uint4*)(Vh + row_of(r) * KC_D + piece * 8) : make_uint4(0u, 0u, 0u, 0u);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const uint32_t w4[4] = {q[u].x, q[u].y, q[u].z, q[u].w};
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float a = __uint_as_float(w4[i] << 16), b = __uint_as_float(w4[i] & 0xffff0000u);
          s = fmaf(a, a, s); s = fmaf(b, b, s);
        }
        p2 += (double)s;
      }
    }
    for (int off = 32; off > 0; off >>= 1) p2 += __shfl_xor(p2, off);
    if (lane == 0) red[wave] = p2;
    __syncthreads();
    f2 = (red[0] + red[1]) + (red[2] + red[3]);
    __syncthreads();
  }
  // Symmetric diagonal scaling S = D^-1/2 G D^-1/2 (unit diagonal): G - mu I is positive definite iff S - mu D^-1 is,
  // and the scaled matrix no longer carries the spread of the channel magnitudes (a few outlier channels otherwise
  // own the trace, and with it the rounding allowance, while lambda_min sits in the small ones).
  const double thr_rel = (double)max(n, KC_D) * 1.1920928955078125e-07;
  const float mu = (float)(thr_rel * thr_rel * f2);
#pragma unroll
  for (int t = 0; t < 3; ++t) {
    if (t < nt && trb[t] == tcb[t] && has_diag) {
      float v = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) if (i == di) v = acc[t][i];
      isd[tcb[t] * 32 + lr] = __builtin_amdgcn_rsqf(v);            // a zero column gives inf, then NaN pivots: not certified
    }
  }
  __syncthreads();
#pragma unroll
  for (int t = 0; t < 3; ++t) {
    if (t < nt) {
      const float sc_col = isd[tcb[t] * 32 + lr];
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const float4 sr = *(const float4*)&isd[trb[t] * 32 + i4 * 8 + lh * 4];
        acc[t][4 * i4 + 0] *= sr.x * sc_col; acc[t][4 * i4 + 1] *= sr.y * sc_col;
        acc[t][4 * i4 + 2] *= sr.z * sc_col; acc[t][4 * i4 + 3] *= sr.w * sc_col;
      }
      if (trb[t] == tcb[t] && has_diag) {
        const float shift = fmaf(mu, sc_col * sc_col, kCertErr * (float)KC_D);   // mu / G_jj + allowance relative to trace(S) = d
#pragma unroll
        for (int i = 0; i < 16; ++i) if (i == di) acc[t][i] -= shift;
      }
    }
  }

  // ---- LDL^T of G - mu I in registers, four columns per step.  panel[s & 1][row] holds columns 4s .. 4s+3 of
  // the current matrix when step s starts.  Thread r < 128 factors the 4x4 diagonal block (the same arithmetic in
  // every thread, so no broadcast) and turns panel row r into y = L d (a 4-term forward substitution) and L; after a
  // second barrier every wave applies the rank-4 update to its tiles: first to the one tile (per wave) that holds
  // the next four columns, which are then published, then to the rest, so the chain block -> next block only
  // contains one tile update.  A non-positive pivot sets a flag (no early exit: the steps stay free of
  // divergent control flow); entries above the diagonal are carried along and never read.
  f32x16 (&g)[3] = acc;
  auto publish = [&](int k) {                         // columns k .. k+3 (k % 4 == 0) -> panel[(k / 4) & 1]
    const int kb = k >> 5, kc = k & 31;
    float* pw = &panel[(k >> 2) & 1][0][0];
#pragma unroll
    for (int t = 0; t < 3; ++t) {
      if (t < nt && tcb[t] == kb && (lr & ~3) == kc) {
        const int c = lr & 3;
#pragma unroll
        for (int i = 0; i < 16; ++i) pw[(trb[t] * 32 + (i >> 2) * 8 + lh * 4 + (i & 3)) * 4 + c] = g[t][i];
      }
    }
  };
  if (tid == 0) s_bad = 0;
  publish(0);
  for (int k = 0; k < KC_D; k += 4) {
    __syncthreads();                                   // this panel visible; ypan / lpan free again
    if (tid < KC_D) {
      const float4* pr = (const float4*)&panel[(k >> 2) & 1][0][0];
      // 4x4 diagonal block: rows k .. k+3, lower triangle
      const float4 r0 = pr[k], r1 = pr[k + 1], r2 = pr[k + 2], r3 = pr[k + 3];
      const float4 x = pr[tid];
      const float d0 = r0.x;
      const float i0 = __builtin_amdgcn_rcpf(d0);
      const float l10 = r1.x * i0, l20 = r2.x * i0, l30 = r3.x * i0;
      const float d1 = fmaf(-l10, r1.x, r1.y);
      const float i1 = __builtin_amdgcn_rcpf(d1);
      const float l21 = fmaf(-l20, r1.x, r2.y) * i1, l31 = fmaf(-l30, r1.x, r3.y) * i1;
      const float y21 = l21 * d1, y31 = l31 * d1;
      const float d2 = fmaf(-l21, y21, fmaf(-l20, r2.x, r2.z));
      const float i2 = __builtin_amdgcn_rcpf(d2);
      const float l32 = fmaf(-l31, y21, fmaf(-l30, r2.x, r3.z)) * i2;
      const float y32 = l32 * d2;
      const float d3 = fmaf(-l32, y32, fmaf(-l31, y31, fmaf(-l30, r3.x, r3.w)));
      const float i3 = __builtin_amdgcn_rcpf(d3);
      if (!((d0 > 0.f) && (d1 > 0.f) && (d2 > 0.f) && (d3 > 0.f))) s_bad = 1;
      // y = L d of panel row x: y0 = x0, y1 = x1 - y0 l10, y2 = x2 - y0 l20 - y1 l21, y3 = x3 - y0 l30 - y1 l31 - y2 l32
      const float y0 = x.x;
      const float y1 = fmaf(-y0, l10, x.y);
      const float y2 = fmaf(-y1, l21, fmaf(-y0, l20, x.z));
      const float y3 = fmaf(-y2, l32, fmaf(-y1, l31, fmaf(-y0, l30, x.w)));
      ypan[tid] = make_float4(y0, y1, y2, y3);
      lpan[tid] = make_float4(y0 * i0, y1 * i1, y2 * i2, y3 * i3);
    }
    __syncthreads();
    const int kb = k >> 5;
    const int kbn = (k + 4) >> 5;                      // column block of the next four columns
    // rank-4 update of a tile on the matrix cores in fp32: G_tile -= Y_rows (32 x 4) * L_cols^T (4 x 32), two
    // v_mfma_f32_32x32x2_f32 (A: lane l holds row l%32, k = l/32; B: k = l/32, column l%32)
    auto update = [&](int t) {
      const float* yp = (const float*)ypan + (trb[t] * 32 + lr) * 4 + lh;
      const float* lp = (const float*)lpan + (tcb[t] * 32 + lr) * 4 + lh;
      const float y0 = -yp[0], y1 = -yp[2], l0 = lp[0], l1 = lp[2];
      g[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(y0, l0, g[t], 0, 0, 0);
      g[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(y1, l1, g[t], 0, 0, 0);
    };
#pragma unroll
    for (int t = 0; t < 3; ++t)
      if (t < nt && tcb[t] == kbn && tcb[t] >= kb) update(t);
    if (k + 4 < KC_D) publish(k + 4);
#pragma unroll
    for (int t = 0; t < 3; ++t)
      if (t < nt && tcb[t] != kbn && tcb[t] >= kb) update(t);
  }
  __syncthreads();
  const bool ok = (s_bad == 0);
  if (!ok) return;

  // certified: r = d, OBF is the identity on this head; fill in the demand sums (Eq. 6) for the diagnostics
  double pk = 0.0, ptot = 0.0;
#pragma unroll
  for (int u = 0; u < 8; ++u) pk += (double)ev[u];
  for (int i0 = tid + 8 * KC_THREADS; i0 < ns; i0 += 8 * KC_THREADS) {      // further batches of index -> score loads
    int j[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) { const int i = i0 + u * KC_THREADS; j[u] = (i < ns) ? id[i] : -1; }
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = (j[u] >= 0) ? sc[j[u]] : 0.f;
#pragma unroll
    for (int u = 0; u < 8; ++u) pk += (double)v[u];
  }
  if (vec_scores) {
    const float4* sc4 = (const float4*)sc;
    const int n4 = Ns >> 2;
    for (int i0 = tid; i0 < n4; i0 += 8 * KC_THREADS) {
      float4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) { const int i = i0 + u * KC_THREADS; v[u] = (i < n4) ? sc4[i] : make_float4(0.f, 0.f, 0.f, 0.f); }
#pragma unroll
      for (int u = 0; u < 8; ++u) ptot += ((double)v[u].x + (double)v[u].y) + ((double)v[u].z + (double)v[u].w);
    }
  } else {
    for (int i = tid; i < Ns; i += KC_THREADS) ptot += (double)sc[i];
  }
  for (int off = 32; off > 0; off >>= 1) { pk += __shfl_xor(pk, off); ptot += __shfl_xor(ptot, off); }
  if (lane == 0) { red[wave] = pk; red2[wave] = ptot; }
  __syncthreads();
  if (tid == 0) {
    const double a_keep = ((red[0] + red[1]) + red[2]) + red[3];
    const double a_tot = ((red2[0] + red2[1]) + red2[2]) + red2[3];
    HeadState s;
    s.a_keep = a_keep; s.a_del = fmax(a_tot - a_keep, 0.0); s.n_keep = n; s.n_del = n_del; s.r_keep = KC_D; s.active = 0;
    s.k_used = 0; s.pad = 0; s.rcr = 0.f; s.ivn = 0.f;
    state[head] = s;
    decided[head] = 1;
  }
}

bool keep_cert_supported(const Dims& m) { return m.dtype == OBF_BF16 && m.d == KC_D; }

obf_status_t launch_keep_cert(const Dims& m, const void* Vsrc, int via_idx, const float* scores, const int32_t* idx,
                              const int32_t* n_keep, int32_t max_budget, int32_t rank, HeadState* state,
                              int32_t* decided, hipStream_t st, const double* fro_part, bool want_sums) {
  const int fro_blocks = (max_budget + kGatherRows - 1) / kGatherRows;
  { ProfScope prof_(ST_KEEP_CERT, st);
    if (via_idx)
      hipLaunchKernelGGL(k_bf_keep_cert<true>, dim3(m.heads), dim3(KC_THREADS), 0, st, (const uint16_t*)Vsrc, scores, idx,
                         n_keep, m.N, max_budget, rank, state, decided, fro_part, fro_blocks, m.scs, m.kvs, want_sums ? 1 : 0);
    else
      hipLaunchKernelGGL(k_bf_keep_cert<false>, dim3(m.heads), dim3(KC_THREADS), 0, st, (const uint16_t*)Vsrc, scores, idx,
                         n_keep, m.N, max_budget, rank, state, decided, fro_part, fro_blocks, m.scs, m.kvs, want_sums ? 1 : 0); }
  return check_launch("backfill keep_cert");
}

}  // namespace obf
