// The message an agent hands on (Sec. 3.3): M_i = [M_{i-1}; Phi(P; G); G] per (layer, KV head), for keys and values:
// a ragged row concatenation of three parts, bit copies in 16-byte pieces, rows behind the message zeroed.
#include "common.hpp"

namespace obf {

constexpr int MS_THREADS = 256;

struct MsgPart { const uint4* K; const uint4* V; int stride; };

__global__ __launch_bounds__(MS_THREADS) void k_append_message(MsgPart prev, const int32_t* __restrict__ prev_len, int prev_len_all,
                                                               MsgPart keep, const int32_t* __restrict__ n_keep,
                                                               MsgPart gen, int n_gen,
                                                               uint4* __restrict__ msg_K, uint4* __restrict__ msg_V,
                                                               int32_t* __restrict__ msg_len, int msg_stride, int row_vec) {
  const int head = blockIdx.y;
  const int rows_per_block = MS_THREADS / row_vec;
  const int r = blockIdx.x * rows_per_block + threadIdx.x / row_vec;
  const int c = threadIdx.x % row_vec;
  const int pl = prev_len ? prev_len[head] : prev_len_all;
  const int nk = n_keep ? n_keep[head] : 0;
  const int total = pl + nk + n_gen;
  // lengths come from the device: a head whose parts do not fit their buffers is left empty and flagged
  const bool fits = pl >= 0 && nk >= 0 && pl <= prev.stride && nk <= keep.stride && total <= msg_stride;
  if (blockIdx.x == 0 && threadIdx.x == 0) msg_len[head] = fits ? total : -1;
  if (r >= msg_stride) return;
  uint4 kv = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
  if (fits && r < total) {
    const MsgPart& p = (r < pl) ? prev : (r < pl + nk) ? keep : gen;
    const int row = (r < pl) ? r : (r < pl + nk) ? r - pl : r - pl - nk;
    const size_t s = ((size_t)head * p.stride + row) * row_vec + c;
    kv = p.K[s];
    vv = p.V[s];
  }
  const size_t o = ((size_t)head * msg_stride + r) * row_vec + c;
  msg_K[o] = kv;
  msg_V[o] = vv;
}

obf_status_t launch_append_message(int heads, int row_bytes, const void* prev_K, const void* prev_V, const int32_t* prev_len,
                                   int prev_len_all, int prev_stride, const void* keep_K, const void* keep_V,
                                   const int32_t* n_keep, int keep_stride, const void* gen_K, const void* gen_V, int n_gen,
                                   int gen_stride, void* msg_K, void* msg_V, int32_t* msg_len, int msg_stride, hipStream_t st) {
  const int row_vec = row_bytes / 16;                    // 8, 16 or 32
  const int rows_per_block = MS_THREADS / row_vec;
  MsgPart prev{(const uint4*)prev_K, (const uint4*)prev_V, prev_stride};
  MsgPart keep{(const uint4*)keep_K, (const uint4*)keep_V, keep_stride};
  MsgPart gen{(const uint4*)gen_K, (const uint4*)gen_V, gen_stride};
  dim3 grid((msg_stride + rows_per_block - 1) / rows_per_block, heads);
  hipLaunchKernelGGL(k_append_message, grid, dim3(MS_THREADS), 0, st, prev, prev_len, prev_len_all, keep, n_keep, gen, n_gen,
                     (uint4*)msg_K, (uint4*)msg_V, msg_len, msg_stride, row_vec);
  return check_launch("append message");
}

}  // namespace obf
