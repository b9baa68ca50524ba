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
// Two launches: (1) the maximum and the normaliser of each of the 2*gamma+1 logit rows of each
// sequence, one workgroup per row; (2) one workgroup per sequence takes the decisions and draws
// the bonus token with a block-wide scan over the vocabulary.  The work is 2 passes over
// (2*gamma+1) * V floats per sequence, once per drafting-verification iteration.
#include "kernels.h"

namespace es {

constexpr int kAcceptThreads = 1024;

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

// stats: [batch][2*gamma+1][2] = (row maximum, sum_v exp((logit_v - maximum) / T)); rows 0..gamma
// are the target's, rows gamma+1..2*gamma the draft's.
__global__ __launch_bounds__(kAcceptThreads) void accept_stats_kernel(const float* __restrict__ draft_logits,
                                                                       const float* __restrict__ target_logits, int gamma, int V,
                                                                       double T, double* __restrict__ stats) {
  __shared__ double sh_d[kAcceptThreads / 64];
  __shared__ float sh_f[kAcceptThreads / 64];
  const int j = blockIdx.x, b = blockIdx.y;
  const float* row = j <= gamma ? target_logits + ((size_t)b * (gamma + 1) + j) * V
                                : draft_logits + ((size_t)b * gamma + (j - gamma - 1)) * V;
  float mx = -INFINITY;
  for (int v = threadIdx.x; v < V; v += blockDim.x) mx = fmaxf(mx, row[v]);
  mx = block_max(mx, sh_f);
  double z = 0.0;
  for (int v = threadIdx.x; v < V; v += blockDim.x) z += exp(((double)row[v] - (double)mx) / T);
  z = block_sum(z, sh_d);
  if (threadIdx.x == 0) {
    double* o = stats + ((size_t)b * (2 * gamma + 1) + j) * 2;
    o[0] = (double)mx;
    o[1] = z;
  }
}

struct BonusDist {
  const float* t;   // target row
  const float* d;   // draft row, or null (plain target distribution)
  double tm, tz, dm, dz, T;
  __device__ __forceinline__ double operator()(int v) const {
    const double p = exp(((double)t[v] - tm) / T) / tz;
    if (!d) return p;
    const double q = p - exp(((double)d[v] - dm) / T) / dz;
    return q > 0.0 ? q : 0.0;
  }
};

__global__ __launch_bounds__(kAcceptThreads) void accept_decide_kernel(const int32_t* __restrict__ draft,
                                                                        const float* __restrict__ draft_logits,
                                                                        const float* __restrict__ target_logits,
                                                                        const float* __restrict__ r, const float* __restrict__ u,
                                                                        int gamma, int V, double T, const double* __restrict__ stats,
                                                                        int32_t* __restrict__ accept_len, int32_t* __restrict__ bonus) {
  __shared__ double sh_d[kAcceptThreads / 64];
  __shared__ double s_incl[kAcceptThreads];
  __shared__ int s_m, s_pick;
  const int b = blockIdx.x, tid = threadIdx.x;
  const double* st = stats + (size_t)b * (2 * gamma + 1) * 2;
  const float* tl = target_logits + (size_t)b * (gamma + 1) * V;
  const float* dl = draft_logits + (size_t)b * gamma * V;
  if (tid == 0) {
    int m = 0;
    for (; m < gamma; ++m) {
      const int x = draft[(size_t)b * gamma + m];
      if (x < 0 || x >= V) { m = -1; break; }  // not a token: reported as accept_len = bonus = -1
      const double p = exp(((double)tl[(size_t)m * V + x] - st[2 * m]) / T) / st[2 * m + 1];
      const double pd = exp(((double)dl[(size_t)m * V + x] - st[2 * (gamma + 1 + m)]) / T) / st[2 * (gamma + 1 + m) + 1];
      if ((double)r[(size_t)b * gamma + m] * pd > p) break;
    }
    s_m = m;
    s_pick = -1;
  }
  __syncthreads();
  const int m = s_m;
  if (m < 0) {
    if (tid == 0) { accept_len[b] = -1; bonus[b] = -1; }
    return;
  }
  BonusDist q;
  q.t = tl + (size_t)m * V;
  q.tm = st[2 * m]; q.tz = st[2 * m + 1]; q.T = T;
  q.d = m < gamma ? dl + (size_t)m * V : nullptr;
  q.dm = m < gamma ? st[2 * (gamma + 1 + m)] : 0.0;
  q.dz = m < gamma ? st[2 * (gamma + 1 + m) + 1] : 1.0;

  // each thread owns a contiguous run of the vocabulary, so that the running sum is in index order
  const int seg = (V + (int)blockDim.x - 1) / (int)blockDim.x;
  const int v0 = min(V, tid * seg), v1 = min(V, v0 + seg);
  double mine = 0.0;
  for (int v = v0; v < v1; ++v) mine += q(v);
  double total = block_sum(mine, sh_d);
  if (q.d && !(total > 0.0)) {
    // identical distributions leave no residual (a rejection is then impossible for r < 1): fall
    // back to the target distribution of that position
    q.d = nullptr;
    mine = 0.0;
    for (int v = v0; v < v1; ++v) mine += q(v);
    total = block_sum(mine, sh_d);
  }
  // inclusive scan of the per-thread sums (Hillis-Steele over LDS; 1024 entries, 10 rounds)
  s_incl[tid] = mine;
  __syncthreads();
  for (int off = 1; off < (int)blockDim.x; off <<= 1) {
    const double add = tid >= off ? s_incl[tid - off] : 0.0;
    __syncthreads();
    s_incl[tid] += add;
    __syncthreads();
  }
  const double thr = (double)u[b] * total;
  const double incl = s_incl[tid], excl = tid ? s_incl[tid - 1] : 0.0;
  if (excl <= thr && thr < incl) {
    // the draw lands in this thread's run; at most one thread gets here (incl is non-decreasing)
    double run = excl;
    int pick = -1, last_pos = v0;
    for (int v = v0; v < v1; ++v) {
      const double qv = q(v);
      if (qv > 0.0) last_pos = v;
      run += qv;
      if (run > thr) { pick = v; break; }
    }
    s_pick = pick >= 0 ? pick : last_pos;  // the scan and the walk may differ in the last bit
  }
  __syncthreads();
  if (tid == 0) {
    int pick = s_pick;
    if (pick < 0) {
      // u * total rounded up to the total: take the last token with positive mass
      pick = V - 1;
      while (pick > 0 && !(q(pick) > 0.0)) --pick;
    }
    accept_len[b] = m;
    bonus[b] = pick;
  }
}

void launch_sample_accept(const int32_t* draft, const float* draft_logits, const float* target_logits, const float* r,
                          const float* u, int batch, int gamma, int V, double T, double* stats, int32_t* accept_len,
                          int32_t* bonus, hipStream_t st) {
  hipLaunchKernelGGL(accept_stats_kernel, dim3(2 * gamma + 1, batch), dim3(kAcceptThreads), 0, st, draft_logits, target_logits,
                     gamma, V, T, stats);
  hipLaunchKernelGGL(accept_decide_kernel, dim3(batch), dim3(kAcceptThreads), 0, st, draft, draft_logits, target_logits, r, u, gamma,
                     V, T, stats, accept_len, bonus);
}

}  // namespace es
