// Small kernels around the hot path (gfx950): weight repacking at load, greedy acceptance, KV cache
// import / export, the streaming-read probe; and their launch wrappers.
#include "launch_common.hpp"

namespace es {

// ------------------------------------------------------------------------------------------
// Small utilities.
// ------------------------------------------------------------------------------------------

// Row-major [.][K] -> tiles of R <= 16 rows, per k-tile a fragment of [k-group 4][R rows] 16-byte
// pieces (1 KB for R = 16: piece i is lane i's share of an MFMA A operand); rows padded with zeros
// up to a multiple of R.  Packed row r is source row r (half = 0), or, for the rotary halves of
// stacked heads (half > 0), source row (r / half) * 2 * half + r % half + row_add: the first
// (row_add = 0) or second (row_add = half) half of head r / half.
template <typename T>
__global__ void repack_kernel(const T* __restrict__ src, u32x4* __restrict__ dst, int rows, int K, int R, int half, int row_add,
                              size_t n_frag) {
  constexpr int EPL = Tr<T>::EPL, KT = Tr<T>::KT;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_frag) return;
  const int nkt = K / KT;
  const int piece = (int)(i % (4 * R));
  const size_t tile = i / (4 * R);
  const int kt = (int)(tile % nkt);
  const size_t rt = tile / nkt;
  const size_t row = rt * R + piece % R;
  u32x4 v = {0u, 0u, 0u, 0u};
  if (row < (size_t)rows) {
    const size_t srow = half > 0 ? (row / half) * 2 * half + row % half + row_add : row;
    v = *reinterpret_cast<const u32x4*>(src + srow * K + (size_t)kt * KT + (piece / R) * EPL);
  }
  dst[i] = v;
}

__global__ void accept_kernel(const int32_t* draft, const int32_t* target, int batch, int gamma, int32_t* accept_len,
                              int32_t* bonus) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= batch) return;
  int m = 0;
  while (m < gamma && draft[b * gamma + m] == target[b * (gamma + 1) + m]) ++m;
  accept_len[b] = m;
  bonus[b] = target[b * (gamma + 1) + m];
}

// user [L][Hkv][n][hd] <-> cache [L][B][Hkv][max_ctx][hd], 16-byte fragments
__global__ void kv_copy_kernel(u32x4* cache, u32x4* user, int L, int B, int Hkv, int max_ctx, int n, int frag_per_row,
                               int seq, int to_cache) {
  const size_t total = (size_t)L * Hkv * n * frag_per_row;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int f = (int)(i % frag_per_row);
  size_t r = i / frag_per_row;
  const int s = (int)(r % n);
  r /= n;
  const int h = (int)(r % Hkv);
  const int l = (int)(r / Hkv);
  const size_t ci = ((((size_t)l * B + seq) * Hkv + h) * max_ctx + s) * frag_per_row + f;
  if (to_cache) cache[ci] = user[i];
  else user[i] = cache[ci];
}

void launch_repack(int dtype, const void* src, void* dst, int rows, int K, int R, int half, int row_add, hipStream_t st) {
  const size_t n_frag = tile_stride(rows, K, dtype, R);
  const unsigned grid = (unsigned)((n_frag + 255) / 256);
  DISPATCH_T(dtype, hipLaunchKernelGGL(repack_kernel<T>, dim3(grid), dim3(256), 0, st, (const T*)src, (u32x4*)dst, rows, K, R, half,
                                       row_add, n_frag));
}
// Streaming-read probe: the same non-temporal 16-byte loads as the weight stream, 8 in flight per
// lane, summed so that nothing is optimised away.  sink: one float per workgroup.
constexpr int kProbeBlocks = 4096, kProbeThreads = 256;
__global__ __launch_bounds__(kProbeThreads) void stream_read_kernel(const u32x4* __restrict__ p, size_t n16, float* sink) {
  // a workgroup reads 8 consecutive 4 KB pieces (32 KB contiguous) per round, as the waves of a
  // weight-streaming workgroup do
  const size_t stride = (size_t)gridDim.x * blockDim.x * 8;
  size_t i = (size_t)blockIdx.x * blockDim.x * 8 + threadIdx.x;
  uint32_t acc = 0;
  for (; i + 7 * (size_t)blockDim.x < n16; i += stride) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(p + i + (size_t)u * blockDim.x);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (int u = 0; u < 8; ++u) {  // ragged end: the last, partial round
    const size_t j = i + (size_t)u * blockDim.x;
    if (j < n16) {
      const u32x4 v = __builtin_nontemporal_load(p + j);
      acc += v.x ^ v.y ^ v.z ^ v.w;
    }
  }
  __shared__ uint32_t sh[kProbeThreads / 64];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) sink[blockIdx.x] = (float)(sh[0] + sh[1] + sh[2] + sh[3]);
}

void launch_stream_read(const void* buf, size_t bytes, float* sink, hipStream_t st) {
  hipLaunchKernelGGL(stream_read_kernel, dim3(kProbeBlocks), dim3(kProbeThreads), 0, st, (const u32x4*)buf, bytes / 16, sink);
}
int stream_read_sink_floats() { return kProbeBlocks; }

void launch_accept(const int32_t* draft, const int32_t* target, int batch, int gamma, int32_t* accept_len, int32_t* bonus,
                   hipStream_t st) {
  hipLaunchKernelGGL(accept_kernel, dim3((batch + 63) / 64), dim3(64), 0, st, draft, target, batch, gamma, accept_len, bonus);
}

void launch_kv_copy(const Shape& s, const Buffers& b, int seq, void* k_user, void* v_user, int n_slots, int to_cache,
                    hipStream_t st) {
  const int fpr = s.hd * (s.dtype == 1 ? 2 : 4) / 16;
  const size_t total = (size_t)s.L * s.Hkv * n_slots * fpr;
  if (total == 0) return;
  const unsigned grid = (unsigned)((total + 255) / 256);
  hipLaunchKernelGGL(kv_copy_kernel, dim3(grid), dim3(256), 0, st, (u32x4*)b.kc, (u32x4*)k_user, s.L, s.B, s.Hkv, s.max_ctx,
                     n_slots, fpr, seq, to_cache);
  hipLaunchKernelGGL(kv_copy_kernel, dim3(grid), dim3(256), 0, st, (u32x4*)b.vc, (u32x4*)v_user, s.L, s.B, s.Hkv, s.max_ctx,
                     n_slots, fpr, seq, to_cache);
}

}  // namespace es
