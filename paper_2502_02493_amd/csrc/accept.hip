// Acceptance by speculative sampling (paper Alg. 3; bonus distribution of Sec. 2.1) on the
// device, in double precision: the decisions (accept or reject, which token the bonus draw
// lands on) are integers decided by floating-point comparisons, so the arithmetic is kept wide
// enough that summation order cannot move a decision except within ~1e-13 of its threshold.
//
//   p'_i = softmax(draft_logits[i] / T),  p_i = softmax(target_logits[i] / T)
//   position i is rejected when r_i * p'_i(x'_i) > p_i(x'_i);  m = first rejected position or gamma
//   bonus ~ max(0, p_m - p'_m) / sum  (m < gamma),  p_gamma  (m = gamma), drawn by inverse CDF in
//   index order with the given uniform u: the lowest v whose running sum exceeds u * sum.
//
// Three launches, all spread over the vocabulary so that no single workgroup has to evaluate
// 10^5 double-precision exponentials:
//   (1) accept_stats_kernel    per logit row and vocabulary slice: slice maximum and
//                              sum exp((l - max) / T)  (combined by the readers);
//   (2) accept_weights_kernel  every workgroup repeats the gamma accept decisions (a few dozen
//                              exponentials), then writes the unnormalised bonus weights q(v) of its
//                              vocabulary chunk and the chunk's sum;
//   (3) accept_draw_kernel     one workgroup per sequence: running sum over the chunk sums in
//                              index order, then inside the chunk the draw lands in.
#include "kernels.h"

#include <mutex>

namespace es {

constexpr int kStatSlices = 8;     // workgroups per logit row in (1)
constexpr int kChunk = 2048;       // vocabulary entries per workgroup in (2) = 2 per thread in (3)
constexpr int kAcceptThreads = 256;
constexpr int kDrawThreads = kChunk / 2;

__device__ __forceinline__ double block_sum(double v, double* sh) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  __syncthreads();  // sh may still be read from the previous call
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  double t = 0.0;
  for (int w = 0; w < (int)(blockDim.x >> 6); ++w) t += sh[w];  // fixed order: same bits in every thread
  return t;
}

__device__ __forceinline__ float block_max(float v, float* sh) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  __syncthreads();
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  float t = -INFINITY;
  for (int w = 0; w < (int)(blockDim.x >> 6); ++w) t = fmaxf(t, sh[w]);
  return t;
}

// Workspace of one sequence (doubles): [rows][kStatSlices][2] slice statistics, then one double
// per vocabulary chunk (chunk sums), then q[V], then one slot holding m.
struct AcceptWs {
  double* stats;
  double* chunk_sum;
  double* q;
  double* m_slot;
};
__host__ __device__ inline size_t accept_ws_doubles(int gamma, int V) {
  const size_t rows = 2 * (size_t)gamma + 1, nchunk = ((size_t)V + kChunk - 1) / kChunk;
  return rows * kStatSlices * 2 + nchunk + (size_t)V + 1;
}
__device__ __forceinline__ AcceptWs accept_ws(double* base, int b, int gamma, int V) {
  const size_t rows = 2 * (size_t)gamma + 1, nchunk = ((size_t)V + kChunk - 1) / kChunk;
  AcceptWs w;
  w.stats = base + (size_t)b * accept_ws_doubles(gamma, V);
  w.chunk_sum = w.stats + rows * kStatSlices * 2;
  w.q = w.chunk_sum + nchunk;
  w.m_slot = w.q + V;
  return w;
}

// rows 0..gamma are the target's, rows gamma+1..2*gamma the draft's.  grid (kStatSlices, rows, batch)
__global__ __launch_bounds__(kAcceptThreads) void accept_stats_kernel(const float* __restrict__ draft_logits,
                                                                       const float* __restrict__ target_logits, int gamma, int V,
                                                                       double T, double* __restrict__ ws) {
  __shared__ double sh_d[kAcceptThreads / 64];
  __shared__ float sh_f[kAcceptThreads / 64];
  const int slice = blockIdx.x, j = blockIdx.y, b = blockIdx.z;
  const float* row = j <= gamma ? target_logits + ((size_t)b * (gamma + 1) + j) * V
                                : draft_logits + ((size_t)b * gamma + (j - gamma - 1)) * V;
  const int per = (V + kStatSlices - 1) / kStatSlices;
  const int v0 = min(V, slice * per), v1 = min(V, v0 + per);
  float mx = -INFINITY;
  for (int v = v0 + threadIdx.x; v < v1; v += blockDim.x) mx = fmaxf(mx, row[v]);
  mx = block_max(mx, sh_f);
  double z = 0.0;
  for (int v = v0 + threadIdx.x; v < v1; v += blockDim.x) z += exp(((double)row[v] - (double)mx) / T);
  z = block_sum(z, sh_d);
  if (threadIdx.x == 0) {
    double* o = accept_ws(ws, b, gamma, V).stats + ((size_t)j * kStatSlices + slice) * 2;
    o[0] = (double)mx;  // -inf for an empty slice; its sum is 0
    o[1] = z;
  }
}

// maximum and normaliser of a row from its slice statistics (slices in order)
__device__ __forceinline__ void row_stats(const double* stats, int row, double T, double* mx, double* z) {
  const double* s = stats + (size_t)row * kStatSlices * 2;
  double m = s[0];
  for (int i = 1; i < kStatSlices; ++i) m = fmax(m, s[2 * i]);
  double t = 0.0;
  for (int i = 0; i < kStatSlices; ++i)
    if (s[2 * i + 1] > 0.0) t += s[2 * i + 1] * exp((s[2 * i] - m) / T);
  *mx = m;
  *z = t;
}

// grid (chunks, batch).  Every workgroup takes the same decisions from the same numbers.
__global__ __launch_bounds__(kAcceptThreads) void accept_weights_kernel(const int32_t* __restrict__ draft,
                                                                         const float* __restrict__ draft_logits,
                                                                         const float* __restrict__ target_logits,
                                                                         const float* __restrict__ r, int gamma, int V, double T,
                                                                         double* __restrict__ ws_base) {
  __shared__ double sh_d[kAcceptThreads / 64];
  __shared__ double s_par[4];
  __shared__ int s_m;
  const int chunk = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const AcceptWs ws = accept_ws(ws_base, b, gamma, V);
  const float* tl = target_logits + (size_t)b * (gamma + 1) * V;
  const float* dl = draft_logits + (size_t)b * gamma * V;
  if (tid == 0) {
    int m = 0;
    double tm = 0.0, tz = 1.0, dm = 0.0, dz = 1.0;
    for (; m < gamma; ++m) {
      const int x = draft[(size_t)b * gamma + m];
      if (x < 0 || x >= V) { m = -1; break; }  // not a token: reported as accept_len = bonus = -1
      row_stats(ws.stats, m, T, &tm, &tz);
      row_stats(ws.stats, gamma + 1 + m, T, &dm, &dz);
      const double p = exp(((double)tl[(size_t)m * V + x] - tm) / T) / tz;
      const double pd = exp(((double)dl[(size_t)m * V + x] - dm) / T) / dz;
      if ((double)r[(size_t)b * gamma + m] * pd > p) break;
    }
    if (m == gamma) row_stats(ws.stats, gamma, T, &tm, &tz);
    s_m = m;
    s_par[0] = tm; s_par[1] = tz; s_par[2] = dm; s_par[3] = dz;
    if (chunk == 0) *ws.m_slot = (double)m;
  }
  __syncthreads();
  const int m = s_m;
  if (m < 0) return;
  const double tm = s_par[0], tz = s_par[1], dm = s_par[2], dz = s_par[3];
  const float* trow = tl + (size_t)m * V;
  const float* drow = m < gamma ? dl + (size_t)m * V : nullptr;
  // each thread owns a contiguous run, so that every sum below is in index order
  constexpr int PER = kChunk / kAcceptThreads;
  const int v0 = chunk * kChunk + tid * PER;
  double mine = 0.0;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int v = v0 + i;
    if (v < V) {
      double q = exp(((double)trow[v] - tm) / T) / tz;
      if (drow) {
        q -= exp(((double)drow[v] - dm) / T) / dz;
        q = q > 0.0 ? q : 0.0;
      }
      ws.q[v] = q;
      mine += q;
    }
  }
  const double tot = block_sum(mine, sh_d);
  if (tid == 0) ws.chunk_sum[chunk] = tot;
}

// grid (batch), kDrawThreads threads (two vocabulary entries each inside the chosen chunk).
__global__ __launch_bounds__(kDrawThreads) void accept_draw_kernel(const float* __restrict__ target_logits,
                                                                    const float* __restrict__ u, int gamma, int V, double T,
                                                                    double* __restrict__ ws_base, int32_t* __restrict__ accept_len,
                                                                    int32_t* __restrict__ bonus) {
  __shared__ double s_incl[kDrawThreads];
  __shared__ double s_thr, s_before;
  __shared__ int s_chunk, s_pick;
  const int b = blockIdx.x, tid = threadIdx.x;
  const AcceptWs ws = accept_ws(ws_base, b, gamma, V);
  const int m = (int)*ws.m_slot;
  if (m < 0) {
    if (tid == 0) { accept_len[b] = -1; bonus[b] = -1; }
    return;
  }
  const int nchunk = (V + kChunk - 1) / kChunk;
  double total = 0.0;
  for (int c0 = 0; c0 < nchunk; c0 += kDrawThreads) {  // chunk sums through LDS: loaded side by side, added in order
    s_incl[tid] = c0 + tid < nchunk ? ws.chunk_sum[c0 + tid] : 0.0;
    __syncthreads();
    if (tid == 0)
      for (int c = 0; c < min(kDrawThreads, nchunk - c0); ++c) total += s_incl[c];
    __syncthreads();
  }
  if (tid == 0) {
    if (!(total > 0.0)) {
      // identical distributions leave no residual (a rejection is then impossible for r < 1): fall
      // back to the target distribution of that position, evaluated here (rare, slow, correct)
      double tm, tz;
      row_stats(ws.stats, m, T, &tm, &tz);
      const float* trow = target_logits + ((size_t)b * (gamma + 1) + m) * V;
      total = 0.0;
      for (int c = 0; c < nchunk; ++c) {
        double cs = 0.0;
        for (int v = c * kChunk; v < min(V, (c + 1) * kChunk); ++v) {
          const double q = exp(((double)trow[v] - tm) / T) / tz;
          ws.q[v] = q;
          cs += q;
        }
        ws.chunk_sum[c] = cs;
        total += cs;
      }
    }
    const double thr = (double)u[b] * total;
    double run = 0.0;
    int pick = -1;
    for (int c = 0; c < nchunk; ++c) {
      const double next = run + ws.chunk_sum[c];
      if (next > thr) { pick = c; break; }
      run = next;
    }
    s_thr = thr;
    s_before = run;
    s_chunk = pick;  // -1: u * total rounded up to the total
    s_pick = -1;
  }
  __syncthreads();
  const int chunk = s_chunk;
  if (chunk >= 0) {
    const int v0 = chunk * kChunk + 2 * tid;
    const double q0 = v0 < V ? ws.q[v0] : 0.0, q1 = v0 + 1 < V ? ws.q[v0 + 1] : 0.0;
    s_incl[tid] = q0 + q1;
    __syncthreads();
    for (int off = 1; off < kDrawThreads; off <<= 1) {  // inclusive scan, Hillis-Steele
      const double add = tid >= off ? s_incl[tid - off] : 0.0;
      __syncthreads();
      s_incl[tid] += add;
      __syncthreads();
    }
    const double thr = s_thr;
    const double excl = s_before + (tid ? s_incl[tid - 1] : 0.0), incl = s_before + s_incl[tid];
    if (excl <= thr && thr < incl) s_pick = (excl + q0 > thr || !(q1 > 0.0)) ? v0 : v0 + 1;  // at most one thread
    __syncthreads();
  }
  if (tid == 0) {
    int pick = s_pick;
    if (pick < 0) {
      // the scans disagreed in the last bit, or the threshold reached the total: the last token
      // with positive weight of the chunk (of the vocabulary)
      pick = min(V, chunk >= 0 ? (chunk + 1) * kChunk : V) - 1;
      while (pick > 0 && !(ws.q[pick] > 0.0)) --pick;
    }
    accept_len[b] = m;
    bonus[b] = pick;
  }
}

size_t sample_accept_workspace_bytes(int batch, int gamma, int V) {
  return (size_t)batch * accept_ws_doubles(gamma, V) * sizeof(double);
}

void launch_sample_accept(const int32_t* draft, const float* draft_logits, const float* target_logits, const float* r,
                          const float* u, int batch, int gamma, int V, double T, double* ws, int32_t* accept_len,
                          int32_t* bonus, hipStream_t st) {
  const int nchunk = (V + kChunk - 1) / kChunk;
  hipLaunchKernelGGL(accept_stats_kernel, dim3(kStatSlices, 2 * gamma + 1, batch), dim3(kAcceptThreads), 0, st, draft_logits,
                     target_logits, gamma, V, T, ws);
  hipLaunchKernelGGL(accept_weights_kernel, dim3(nchunk, batch), dim3(kAcceptThreads), 0, st, draft, draft_logits, target_logits, r,
                     gamma, V, T, ws);
  hipLaunchKernelGGL(accept_draw_kernel, dim3(batch), dim3(kDrawThreads), 0, st, target_logits, u, gamma, V, T, ws, accept_len,
                     bonus);
}

// ------------------------------------------------------------------------------------------
// The same three launches for callers that cannot allocate and bring no workspace: the
// workspace is a file-scope device array.  Its name is a host-side stand-in, not a device
// address: the address comes from hipGetSymbolAddress, once per device with that device
// current (every GPU holds its own copy), and only that pointer is handed to kernels.
// ------------------------------------------------------------------------------------------
constexpr size_t kStaticWsDoubles = (size_t)1 << 20;  // 8 MiB per GPU, held until the process ends
static __device__ __align__(256) double scratch[kStaticWsDoubles];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static double* g_scratch_ptr[kMaxDevices];  // per device, filled at the first call on it

size_t sample_accept_static_capacity_bytes() { return kStaticWsDoubles * sizeof(double); }

hipError_t sample_accept_static_workspace(double** out) {
  *out = nullptr;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    double* p = nullptr;
    e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace es
