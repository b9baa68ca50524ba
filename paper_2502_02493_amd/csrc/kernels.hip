// gfx950 (CDNA4, wave64) kernels of the EasySpec draft hot path.
//
// Every weight contraction of the model is the same shape of work: a matrix that is far larger
// than any cache is streamed from HBM exactly once and multiplied with at most 16 token
// columns (1 per live sequence in a fuzzy draft step, paper Alg. 2; the accepted tokens plus
// the bonus token in calibration, paper Sec. 3.2).  All of them therefore share one core:
//
//   * Weights are repacked at load time into 1 KB tiles of 16 rows x KT columns (KT = 32 bf16
//     or 16 fp32).  Inside a tile, lane l of a wavefront owns 16 contiguous bytes: row l%16,
//     columns (l/16)*EPL .. +EPL-1.  That is exactly the A-operand register layout of the
//     16x16 MFMA instructions, so one fully coalesced 1 KB wave load feeds one MFMA with no
//     shuffling, and a row tile's K sweep is one contiguous ascending address stream.
//   * The token columns are the MFMA's N dimension (B operand, 16 bytes per lane read from a
//     small L2-resident activation array, only lanes of live columns load).
//   * The waves of a workgroup split K between them (interleaved, so the workgroup reads
//     consecutive KBs), partial accumulators are summed through LDS in a fixed order, and wave
//     0 runs the epilogue that the operation needs (bias + rotary + cache write, residual
//     update + next norm input, SiLU*up, logits + argmax).
//
// RMSNorm is split so that no kernel has to normalise before it can start streaming: the
// producer of a residual vector h writes T(h * gain) for the consumer's gain and the partial
// sums of squares of h per 16-row tile; the consumer multiplies its accumulators by
// rsqrt(mean(h^2) + eps).  Both sides of the parity tests use this order of roundings.
#include "kernels.h"

#include <algorithm>
#include <type_traits>

namespace es {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct bf16_t {
  uint16_t bits;
};

template <typename T>
struct Tr;
template <>
struct Tr<float> {
  static constexpr int EPL = 4, KT = 16, PARTS = 1;
};
// bf16 activations are carried as two bf16 terms, hi = bf16(x) and lo = bf16(x - hi), stored as
// two arrays [hi | lo]; the contraction runs one MFMA per term.  MFMA issue slots are idle in
// this HBM-bound work, so the second term is free and keeps activations at ~16 mantissa bits.
template <>
struct Tr<bf16_t> {
  static constexpr int EPL = 8, KT = 32, PARTS = 2;
};

// Layout of an activation operand x[col][k] (col < 16, k < K) of a weight contraction, per
// part (hi, lo).  It depends on the number of columns of the forward pass, which producer and
// consumer both know:
//   up to kPlainCols columns: plain rows, x[col][k] at col * K + k.  A wave's B fragments of one
//     k-tile are then one 64-byte run per column: the fewest cache lines for one or two columns.
//   more columns: 1 KB tiles of KT consecutive k, inside a tile [k-group (4)][column (16)][EPL
//     elements] — the order in which the 64 lanes of a wave take their 16-byte fragments (lane =
//     k-group * 16 + column) — so that a fragment load is one contiguous run per k-group and part
//     instead of one cache line per column (measured: 6-column calibration 7 % faster, 8-wide tree
//     level 12 %; with one column the tiles would touch four times the lines of plain rows).
constexpr int kPlainCols = 2;

template <typename T>
__device__ __forceinline__ size_t xoff(int ncols, int K, int col, int k) {
  constexpr int EPL = Tr<T>::EPL, KT = Tr<T>::KT;
  if (ncols <= kPlainCols) return (size_t)col * K + k;
  return (size_t)(k / KT) * (kMaxCols * KT) + (size_t)((k % KT) / EPL) * (kMaxCols * EPL) + col * EPL + (k % EPL);
}
// u32x4 between the fragments of consecutive k-tiles
template <typename T>
__device__ __forceinline__ int xtile_stride(int ncols) {
  return ncols <= kPlainCols ? 4 : 64;
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ uint32_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);  // round to nearest, ties to even
  return u >> 16;
}

template <typename T>
__device__ __forceinline__ float load1(const T* p);
template <>
__device__ __forceinline__ float load1<float>(const float* p) {
  return *p;
}
template <>
__device__ __forceinline__ float load1<bf16_t>(const bf16_t* p) {
  return bf16_bits_to_float(p->bits);
}

template <typename T>
__device__ __forceinline__ void store1(T* p, float v);
template <>
__device__ __forceinline__ void store1<float>(float* p, float v) {
  *p = v;
}
template <>
__device__ __forceinline__ void store1<bf16_t>(bf16_t* p, float v) {
  p->bits = (uint16_t)float_to_bf16_bits(v);
}

// four consecutive elements, p aligned to 4 elements
template <typename T>
__device__ __forceinline__ void store4(T* p, float a, float b, float c, float d);
template <>
__device__ __forceinline__ void store4<float>(float* p, float a, float b, float c, float d) {
  f32x4 v = {a, b, c, d};
  *reinterpret_cast<f32x4*>(p) = v;
}
template <>
__device__ __forceinline__ void store4<bf16_t>(bf16_t* p, float a, float b, float c, float d) {
  u32x2 v = {float_to_bf16_bits(a) | (float_to_bf16_bits(b) << 16), float_to_bf16_bits(c) | (float_to_bf16_bits(d) << 16)};
  *reinterpret_cast<u32x2*>(p) = v;
}

// Activation stores: p points into the "hi" array, the "lo" array starts part elements later.
template <typename T>
__device__ __forceinline__ void store_act1(T* p, size_t part, float v);
template <>
__device__ __forceinline__ void store_act1<float>(float* p, size_t, float v) {
  *p = v;
}
template <>
__device__ __forceinline__ void store_act1<bf16_t>(bf16_t* p, size_t part, float v) {
  const uint32_t hi = float_to_bf16_bits(v);
  p->bits = (uint16_t)hi;
  p[part].bits = (uint16_t)float_to_bf16_bits(v - bf16_bits_to_float(hi));
}
template <typename T>
__device__ __forceinline__ void store_act4(T* p, size_t part, float a, float b, float c, float d);
template <>
__device__ __forceinline__ void store_act4<float>(float* p, size_t, float a, float b, float c, float d) {
  store4<float>(p, a, b, c, d);
}
template <>
__device__ __forceinline__ void store_act4<bf16_t>(bf16_t* p, size_t part, float a, float b, float c, float d) {
  const uint32_t ha = float_to_bf16_bits(a), hb = float_to_bf16_bits(b), hc = float_to_bf16_bits(c), hd = float_to_bf16_bits(d);
  u32x2 hi = {ha | (hb << 16), hc | (hd << 16)};
  *reinterpret_cast<u32x2*>(p) = hi;
  store4<bf16_t>(p + part, a - bf16_bits_to_float(ha), b - bf16_bits_to_float(hb), c - bf16_bits_to_float(hc),
                 d - bf16_bits_to_float(hd));
}

// unpack the EPL elements of one 16-byte fragment
template <typename T>
__device__ __forceinline__ void unpack(const u32x4& r, float (&out)[Tr<T>::EPL]);
template <>
__device__ __forceinline__ void unpack<float>(const u32x4& r, float (&out)[4]) {
  out[0] = __uint_as_float(r.x); out[1] = __uint_as_float(r.y); out[2] = __uint_as_float(r.z); out[3] = __uint_as_float(r.w);
}
template <>
__device__ __forceinline__ void unpack<bf16_t>(const u32x4& r, float (&out)[8]) {
  out[0] = __uint_as_float(r.x << 16); out[1] = __uint_as_float(r.x & 0xFFFF0000u);
  out[2] = __uint_as_float(r.y << 16); out[3] = __uint_as_float(r.y & 0xFFFF0000u);
  out[4] = __uint_as_float(r.z << 16); out[5] = __uint_as_float(r.z & 0xFFFF0000u);
  out[6] = __uint_as_float(r.w << 16); out[7] = __uint_as_float(r.w & 0xFFFF0000u);
}

// One k-tile of multiply-accumulate: acc[16 rows x 16 cols] += A[16 x KT] * B[KT x 16].
template <typename T>
__device__ __forceinline__ void mma(f32x4& acc, const u32x4& a, const u32x4& b);
template <>
__device__ __forceinline__ void mma<bf16_t>(f32x4& acc, const u32x4& a, const u32x4& b) {
  acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}
template <>
__device__ __forceinline__ void mma<float>(f32x4& acc, const u32x4& a, const u32x4& b) {
  // four K=4 steps; step e contracts element e of every lane's fragment (same k on both sides)
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
}

// ------------------------------------------------------------------------------------------
// The shared core.  w[r]: first tile of row tile r (tiles of one row tile are consecutive,
// 64 u32x4 each).  x: activation operand in T (layout: xoff).  The calling wave accumulates k-tiles
// wave, wave+NW, ... into acc.
//
// NB = B fragments (and MFMAs) per weight tile.  With two-term activations and at most 8
// columns, the lo terms ride in MFMA columns ncols..2*ncols-1 of the same instruction
// ("folded", NB = 1) and fold_columns() adds the two halves afterwards; with more columns the
// hi and lo terms take one MFMA each (NB = 2).  A wave keeps one batch of 8 KB in flight; two
// batches per wave were measured slower (the registers cost more occupancy than they hide).
// ------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ bool folded(int ncols) {
  return Tr<T>::PARTS == 2 && 2 * ncols <= kMaxCols;
}

template <typename T, int RT, int NB>
__device__ __forceinline__ void gemm_loop(const u32x4* const (&w)[RT], const u32x4* const (&xp)[NB], int xs, bool colok,
                                          int nkt, f32x4 (&acc)[RT], int w_lane, int w_stride) {
  constexpr int U = 8 / RT;  // k-tiles per batch: 8 KB of weights in flight per wave
  const int wave = threadIdx.x >> 6, NW = blockDim.x >> 6;
  // w_lane: the lane's 16-byte piece of a weight fragment, w_stride: pieces per fragment (lane and 64 for tiles of 16 rows)
  const u32x4* wp[RT];
#pragma unroll
  for (int r = 0; r < RT; ++r) wp[r] = w[r] + w_lane;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  int kt = wave;
  for (; kt + (U - 1) * NW < nkt; kt += U * NW) {
    u32x4 a[RT][U], b[NB][U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int r = 0; r < RT; ++r) a[r][u] = __builtin_nontemporal_load(wp[r] + (size_t)(kt + u * NW) * w_stride);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int q = 0; q < NB; ++q) b[q][u] = colok ? xp[q][(size_t)(kt + u * NW) * xs] : zero;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int r = 0; r < RT; ++r) {
#pragma unroll
        for (int q = 0; q < NB; ++q) mma<T>(acc[r], a[r][u], b[q][u]);
      }
    }
  }
  if (kt < nkt) {
    // last, partial batch: same shape with the loads past the end switched off (wave-uniform), so
    // that the remaining tiles are still fetched together instead of one latency at a time
    u32x4 a[RT][U], b[NB][U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool in = kt + u * NW < nkt;
#pragma unroll
      for (int r = 0; r < RT; ++r) a[r][u] = in ? __builtin_nontemporal_load(wp[r] + (size_t)(kt + u * NW) * w_stride) : zero;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool in = colok && kt + u * NW < nkt;
#pragma unroll
      for (int q = 0; q < NB; ++q) b[q][u] = in ? xp[q][(size_t)(kt + u * NW) * xs] : zero;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int r = 0; r < RT; ++r) {
#pragma unroll
        for (int q = 0; q < NB; ++q) mma<T>(acc[r], a[r][u], b[q][u]);
      }
    }
  }
}

// NB is chosen by the host per launch: 1 when the activations have one term (fp32) or the
// columns fold (at most 8), else 2.  Separate instantiations keep the common one-fragment path
// free of the second path's registers.
template <typename T, int RT, int NB>
__device__ __forceinline__ void gemm_accumulate(const u32x4* const (&w)[RT], const T* __restrict__ x, int K, int ncols,
                                                f32x4 (&acc)[RT], int w_lane = -1, int w_stride = 64) {
  constexpr int EPL = Tr<T>::EPL, KT = Tr<T>::KT, PARTS = Tr<T>::PARTS;
  const int lane = threadIdx.x & 63;
  const int col = lane & 15, kg = lane >> 4;
  const int nkt = K / KT;
  const size_t part = (size_t)kMaxCols * K;  // elements between the hi and lo arrays
  if (w_lane < 0) w_lane = lane;  // full tiles: fragment piece i belongs to lane i
  if (NB == 1) {
    // lane column c < ncols reads the hi term of column c, column ncols + c its lo term
    const bool is_lo = PARTS == 2 && col >= ncols;
    const int src = is_lo ? col - ncols : col;
    const bool colok = src < ncols;
    const u32x4* const xp[1] = {
        reinterpret_cast<const u32x4*>(x + (is_lo ? part : 0) + xoff<T>(ncols, K, colok ? src : 0, kg * EPL))};
    gemm_loop<T, RT, 1>(w, xp, xtile_stride<T>(ncols), colok, nkt, acc, w_lane, w_stride);
  } else {
    const bool colok = col < ncols;
    const T* base = x + xoff<T>(ncols, K, colok ? col : 0, kg * EPL);
    const u32x4* const xp[2] = {reinterpret_cast<const u32x4*>(base), reinterpret_cast<const u32x4*>(base + part)};
    gemm_loop<T, RT, 2>(w, xp, xtile_stride<T>(ncols), colok, nkt, acc, w_lane, w_stride);
  }
}

// After reduce_waves, in the wave that holds the totals: add the lo-term columns onto the
// hi-term columns when the contraction ran folded.  All 64 lanes must call it.
template <typename T, int RT>
__device__ __forceinline__ void fold_columns(f32x4 (&acc)[RT], int ncols) {
  if (!folded<T>(ncols)) return;
#pragma unroll
  for (int r = 0; r < RT; ++r)
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[r][i] += __shfl_down(acc[r][i], ncols, 64);
}

// Sum the waves' partial accumulators through LDS in wave order; true for the wave that holds
// the total (wave 0).  red: (NW-1)*RT*64 f32x4.
template <int RT>
__device__ __forceinline__ bool reduce_waves(f32x4 (&acc)[RT], f32x4* red) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, NW = blockDim.x >> 6;
  if (NW == 1) return true;
  if (wave > 0) {
#pragma unroll
    for (int r = 0; r < RT; ++r) red[((wave - 1) * RT + r) * 64 + lane] = acc[r];
  }
  __syncthreads();
  if (wave == 0) {
    for (int w = 1; w < NW; ++w) {
#pragma unroll
      for (int r = 0; r < RT; ++r) acc[r] += red[((w - 1) * RT + r) * 64 + lane];
    }
  }
  return wave == 0;
}

// rstd[col] = rsqrt(sum_t ssp[col][t] / d + eps), summed in a fixed order.  Ends with a barrier.
__device__ __forceinline__ void compute_rstd(const float* __restrict__ ssp, int ntile, int ncols, float inv_d, float eps,
                                             float* s_rstd) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, NW = blockDim.x >> 6;
  for (int col = wave; col < ncols; col += NW) {
    float s = 0.f;
    for (int t = lane; t < ntile; t += 64) s += ssp[col * ntile + t];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (lane == 0) s_rstd[col] = 1.0f / sqrtf(s * inv_d + eps);
  }
  __syncthreads();
}

// The same quantity with its loads issued BEFORE the weight stream of the workgroup starts and
// its arithmetic done after: the L2 latency of the partial sums then hides behind the stream
// instead of sitting in the tail of the kernel.  Covers d <= 4096 and up to two columns per
// wave (the common cases); otherwise rstd_finish falls back to compute_rstd.  Same summation
// order as compute_rstd, so both give identical bits.
struct RstdPre {
  float v[2][4];
  bool fast;
};

__device__ __forceinline__ void rstd_issue(const float* __restrict__ ssp, int ntile, int ncols, RstdPre& p) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, NW = blockDim.x >> 6;
  p.fast = ntile <= 256 && ncols <= 2 * NW;
  if (!p.fast) return;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int col = wave + i * NW;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int t = lane + 64 * j;
      p.v[i][j] = (col < ncols && t < ntile) ? ssp[col * ntile + t] : 0.f;
    }
  }
}

// Ends with a barrier unless the caller's reduce_waves provides one (NW > 1).
__device__ __forceinline__ void rstd_finish(const float* __restrict__ ssp, int ntile, int ncols, float inv_d, float eps,
                                            const RstdPre& p, float* s_rstd) {
  if (!p.fast) {
    compute_rstd(ssp, ntile, ncols, inv_d, eps, s_rstd);
    return;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, NW = blockDim.x >> 6;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int col = wave + i * NW;
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (lane + 64 * j < ntile) s += p.v[i][j];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (lane == 0 && col < ncols) s_rstd[col] = 1.0f / sqrtf(s * inv_d + eps);
  }
  if (NW == 1) __syncthreads();
}

extern __shared__ f32x4 dyn_red[];

// ------------------------------------------------------------------------------------------
// QKV projection of the k layers of a set + bias + rotary + KV-cache write.
// Unit of work: two row tiles of one head, rows e and e + hd/2, so that the rotation pairs
// sit in the same lane.  grid = k * (Hq + 2 Hkv) * (hd/32).
// ------------------------------------------------------------------------------------------
struct QkvArgs {
  const u32x4* w;  // layer layer0
  size_t w_layer_stride;
  const void* x;  // XA: k operand slots of 16 x d
  const float* ssp;
  const float* bias;  // layer layer0, or null
  const float2* rope;
  float* q;
  void* kc;
  void* vc;
  int layer0, d, Hq, Hkv, hd, B, max_ctx;
  float inv_d, eps;
};

template <typename T, int NB>
__global__ __launch_bounds__(1024) void qkv_kernel(QkvArgs a, Cols c) {
  __shared__ float s_rstd[kMaxCols];
  const int KT = Tr<T>::KT;
  const int nkt = a.d / KT;
  const int pairs = a.hd / 32;
  const int units = (a.Hq + 2 * a.Hkv) * pairs;
  const int li = blockIdx.x / units, u = blockIdx.x % units;
  const int head = u / pairs, p = u % pairs;
  const int rt0 = head * (a.hd / 16) + p, rt1 = rt0 + pairs;
  const u32x4* wl = a.w + (size_t)li * a.w_layer_stride;
  const u32x4* const w[2] = {wl + (size_t)rt0 * nkt * 64, wl + (size_t)rt1 * nkt * 64};
  const T* x = reinterpret_cast<const T*>(a.x) + (size_t)li * Tr<T>::PARTS * kMaxCols * a.d;
  // operands of the epilogue (wave 0 only) and of the norm scale are fetched before the weight
  // stream starts, so that their latency does not sit in the tail of the kernel
  const int lane = threadIdx.x & 63, col = lane & 15;
  const int e0 = p * 16 + (lane >> 4) * 4;  // element inside the head, < hd/2
  const int half = a.hd / 2;
  const int RQKV = (a.Hq + 2 * a.Hkv) * a.hd;
  const bool epi = threadIdx.x < 64 && col < c.n;
  const int pos = epi ? c.pos[col] : 0, seq = epi ? c.seq[col] : 0;
  f32x4 b_lo = {0.f, 0.f, 0.f, 0.f}, b_hi = {0.f, 0.f, 0.f, 0.f}, cs01 = {1.f, 0.f, 1.f, 0.f}, cs23 = {1.f, 0.f, 1.f, 0.f};
  if (epi) {
    if (a.bias) {
      b_lo = *reinterpret_cast<const f32x4*>(a.bias + (size_t)li * RQKV + head * a.hd + e0);
      b_hi = *reinterpret_cast<const f32x4*>(a.bias + (size_t)li * RQKV + head * a.hd + e0 + half);
    }
    if (head < a.Hq + a.Hkv) {
      const f32x4* rp = reinterpret_cast<const f32x4*>(a.rope + (size_t)c.rope_pos[col] * half + e0);  // 4 x (cos, sin)
      cs01 = rp[0];
      cs23 = rp[1];
    }
  }
  RstdPre pre;
  rstd_issue(a.ssp, a.d / 16, c.n, pre);

  f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
  gemm_accumulate<T, 2, NB>(w, x, a.d, c.n, acc);
  rstd_finish(a.ssp, a.d / 16, c.n, a.inv_d, a.eps, pre, s_rstd);
  if (!reduce_waves<2>(acc, dyn_red)) return;
  fold_columns<T, 2>(acc, c.n);

  if (col >= c.n) return;
  const float r = s_rstd[col];
  const float cosv[4] = {cs01[0], cs01[2], cs23[0], cs23[2]}, sinv[4] = {cs01[1], cs01[3], cs23[1], cs23[3]};
  float lo[4], hi[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    // identity rotation (cos 1, sin 0) for the V rows; bias 0 without bias
    const float v0 = acc[0][i] * r + b_lo[i], v1 = acc[1][i] * r + b_hi[i];
    lo[i] = v0 * cosv[i] - v1 * sinv[i];
    hi[i] = v1 * cosv[i] + v0 * sinv[i];
  }
  if (head < a.Hq) {
    float* q = a.q + ((size_t)li * kMaxCols + col) * (a.Hq * a.hd) + head * a.hd + e0;
    store4<float>(q, lo[0], lo[1], lo[2], lo[3]);
    store4<float>(q + half, hi[0], hi[1], hi[2], hi[3]);
  } else {
    const bool is_k = head < a.Hq + a.Hkv;
    const int kvh = is_k ? head - a.Hq : head - a.Hq - a.Hkv;
    T* base = reinterpret_cast<T*>(is_k ? a.kc : a.vc);
    T* row = base + ((((size_t)(a.layer0 + li) * a.B + seq) * a.Hkv + kvh) * a.max_ctx + pos) * a.hd + e0;
    store4<T>(row, lo[0], lo[1], lo[2], lo[3]);
    store4<T>(row + half, hi[0], hi[1], hi[2], hi[3]);
  }
}

// ------------------------------------------------------------------------------------------
// Projection back into the residual stream: the O projections of a set's layers in one
// launch (k > 1), or one down projection (k = 1).  Layer 0 of the launch updates the
// residual: h = H + acc (+ Attnoutput of the next layer), writes H, the sum of squares of h
// and T(h * gain_j) for the consumer(s) that come next; the other layers only store their
// Attnoutput for later.  grid = k * d/16.
// ------------------------------------------------------------------------------------------
struct ProjArgs {
  const u32x4* w;
  size_t w_layer_stride;
  const void* x;  // k operand slots of 16 x K in T
  int K, d;
  float* H;
  float* A;      // [MAX_SET][16][d]
  int a_add;     // slot of A to add to the residual after acc, or -1
  const float* gain;
  int n_gain;
  void* xout;    // n_gain operand slots of 16 x d in T
  float* ssp;
};

template <typename T, int NB>
__global__ __launch_bounds__(1024) void proj_resid_kernel(ProjArgs a, Cols c) {
  const int KT = Tr<T>::KT;
  const int nkt = a.K / KT;
  const int ntile = a.d / 16;
  const int li = blockIdx.x / ntile, t = blockIdx.x % ntile;
  const u32x4* const w[1] = {a.w + (size_t)li * a.w_layer_stride + (size_t)t * nkt * 64};
  const T* x = reinterpret_cast<const T*>(a.x) + (size_t)li * Tr<T>::PARTS * kMaxCols * a.K;
  // residual-update operands (wave 0 of a layer-0 workgroup) are fetched before the weight stream
  const int lane = threadIdx.x & 63, col = lane & 15;
  const bool ok = col < c.n;
  const int r0 = t * 16 + (lane >> 4) * 4;
  f32x4 h_in = {0.f, 0.f, 0.f, 0.f}, a_in = {0.f, 0.f, 0.f, 0.f}, g_in = {0.f, 0.f, 0.f, 0.f};
  if (threadIdx.x < 64 && li == 0 && ok) {
    h_in = *reinterpret_cast<const f32x4*>(a.H + (size_t)col * a.d + r0);
    if (a.a_add >= 0) a_in = *reinterpret_cast<const f32x4*>(a.A + ((size_t)a.a_add * kMaxCols + col) * a.d + r0);
    g_in = *reinterpret_cast<const f32x4*>(a.gain + r0);
  }
  f32x4 acc[1] = {{0.f, 0.f, 0.f, 0.f}};
  gemm_accumulate<T, 1, NB>(w, x, a.K, c.n, acc);
  if (!reduce_waves<1>(acc, dyn_red)) return;
  fold_columns<T, 1>(acc, c.n);

  if (li > 0) {
    if (ok) store4<float>(a.A + ((size_t)li * kMaxCols + col) * a.d + r0, acc[0][0], acc[0][1], acc[0][2], acc[0][3]);
    return;
  }
  float ss = 0.f;
  if (ok) {
    float* hp = a.H + (size_t)col * a.d + r0;
    f32x4 h = h_in;
    h += acc[0];
    if (a.a_add >= 0) h += a_in;
    *reinterpret_cast<f32x4*>(hp) = h;
    for (int j = 0; j < a.n_gain; ++j) {
      const f32x4 g = j == 0 ? g_in : *reinterpret_cast<const f32x4*>(a.gain + (size_t)j * a.d + r0);
      T* xo = reinterpret_cast<T*>(a.xout) + (size_t)j * Tr<T>::PARTS * kMaxCols * a.d + xoff<T>(c.n, a.d, col, r0);
      store_act4<T>(xo, (size_t)kMaxCols * a.d, h[0] * g[0], h[1] * g[1], h[2] * g[2], h[3] * g[3]);
    }
    ss = h[0] * h[0] + h[1] * h[1] + h[2] * h[2] + h[3] * h[3];
  }
  ss += __shfl_xor(ss, 16, 64);
  ss += __shfl_xor(ss, 32, 64);
  if (ok && lane < 16) a.ssp[col * ntile + t] = ss;
}

// ------------------------------------------------------------------------------------------
// The two projections of full-layer-parallel mode (the ablation of App. B: every layer of a set,
// attention and MLP, works from the set's input h_1 = H; the set's output is
// H + sum_i (Attnoutput_i + MLPoutput_i)).
//   down == 0, O projections of the set, grid = k * d/16: layer li parks Attnoutput_li in A[li]
//     and writes the input of its own MLP, T((H + Attnoutput_li) * gain_li), into operand slot li
//     of xout with the partial sums of squares in slot li of ssp; H is left alone.
//   down == 1, down projections of the set, grid = d/16: a workgroup adds up the k layers'
//     contractions for its row tile (operand slot li of x against layer li of w), then
//     h = H + that sum + A[0] + ... + A[k-1]; writes H, the partial sums of squares of h and
//     T(h * gain_j) for the n_gain consumers that come next, like proj_resid_kernel.
// ------------------------------------------------------------------------------------------
struct ProjFullArgs {
  const u32x4* w;
  size_t w_layer_stride;
  const void* x;  // k operand slots of 16 x K in T
  int K, d, k, down;
  float* H;
  float* A;       // [MAX_SET][16][d]
  const float* gain;  // down == 0: [k][d]; down == 1: [n_gain][d]
  int n_gain;
  void* xout;
  float* ssp;     // down == 0: [k][16][d/16]; down == 1: [16][d/16]
};

template <typename T, int NB>
__global__ __launch_bounds__(1024) void proj_full_kernel(ProjFullArgs a, Cols c) {
  const int nkt = a.K / Tr<T>::KT;
  const int ntile = a.d / 16;
  const int li = a.down ? 0 : blockIdx.x / ntile, t = blockIdx.x % ntile;
  const int lane = threadIdx.x & 63, col = lane & 15;
  const bool ok = col < c.n;
  const int r0 = t * 16 + (lane >> 4) * 4;
  f32x4 acc[1] = {{0.f, 0.f, 0.f, 0.f}};
  const int n_sum = a.down ? a.k : 1;
  for (int j = 0; j < n_sum; ++j) {  // uniform over the workgroup
    const int l = li + j;
    const u32x4* const w[1] = {a.w + (size_t)l * a.w_layer_stride + (size_t)t * nkt * 64};
    gemm_accumulate<T, 1, NB>(w, reinterpret_cast<const T*>(a.x) + (size_t)l * Tr<T>::PARTS * kMaxCols * a.K, a.K, c.n, acc);
  }
  if (!reduce_waves<1>(acc, dyn_red)) return;
  fold_columns<T, 1>(acc, c.n);

  float ss = 0.f;
  if (ok) {
    f32x4 h = *reinterpret_cast<const f32x4*>(a.H + (size_t)col * a.d + r0);
    h += acc[0];
    if (a.down) {
      for (int j = 0; j < a.k; ++j) h += *reinterpret_cast<const f32x4*>(a.A + ((size_t)j * kMaxCols + col) * a.d + r0);
      *reinterpret_cast<f32x4*>(a.H + (size_t)col * a.d + r0) = h;
      for (int j = 0; j < a.n_gain; ++j) {
        const f32x4 g = *reinterpret_cast<const f32x4*>(a.gain + (size_t)j * a.d + r0);
        T* xo = reinterpret_cast<T*>(a.xout) + (size_t)j * Tr<T>::PARTS * kMaxCols * a.d + xoff<T>(c.n, a.d, col, r0);
        store_act4<T>(xo, (size_t)kMaxCols * a.d, h[0] * g[0], h[1] * g[1], h[2] * g[2], h[3] * g[3]);
      }
    } else {
      store4<float>(a.A + ((size_t)li * kMaxCols + col) * a.d + r0, acc[0][0], acc[0][1], acc[0][2], acc[0][3]);
      const f32x4 g = *reinterpret_cast<const f32x4*>(a.gain + (size_t)li * a.d + r0);
      T* xo = reinterpret_cast<T*>(a.xout) + (size_t)li * Tr<T>::PARTS * kMaxCols * a.d + xoff<T>(c.n, a.d, col, r0);
      store_act4<T>(xo, (size_t)kMaxCols * a.d, h[0] * g[0], h[1] * g[1], h[2] * g[2], h[3] * g[3]);
    }
    ss = h[0] * h[0] + h[1] * h[1] + h[2] * h[2] + h[3] * h[3];
  }
  ss += __shfl_xor(ss, 16, 64);
  ss += __shfl_xor(ss, 32, 64);
  if (ok && lane < 16) a.ssp[(size_t)li * kMaxCols * ntile + col * ntile + t] = ss;
}

// ------------------------------------------------------------------------------------------
// Gate and up projections + SiLU(gate) * up of one layer, or of the k layers of a set each on
// its own input (full-layer mode): layer li of the launch reads operand slot li of x with
// partial sums slot li and writes operand slot li of act.  grid = k * F/16.
// ------------------------------------------------------------------------------------------
struct GateUpArgs {
  const u32x4* wg;
  const u32x4* wu;
  size_t w_layer_stride;
  const void* x;  // XM: k operand slots of 16 x d
  const float* ssp;  // [k][16][d/16]
  void* act;  // k operand slots of 16 x F in T
  int d, F;
  int R;      // rows per weight tile (tile_rows() of F), ntile = ceil(F / R) workgroups per layer
  float inv_d, eps;
};

template <typename T, int NB>
__global__ __launch_bounds__(1024) void gateup_kernel(GateUpArgs a, Cols c) {
  __shared__ float s_rstd[kMaxCols];
  const int nkt = a.d / Tr<T>::KT;
  const int R = a.R, ntile = (a.F + R - 1) / R;
  const int li = blockIdx.x / ntile, t = blockIdx.x % ntile;
  const size_t wl = (size_t)li * a.w_layer_stride + (size_t)t * nkt * (4 * R);
  const u32x4* const w[2] = {a.wg + wl, a.wu + wl};
  const float* ssp = a.ssp + (size_t)li * kMaxCols * (a.d / 16);
  RstdPre pre;
  rstd_issue(ssp, a.d / 16, c.n, pre);
  f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
  // a tile of R < 16 rows: the lanes of the missing rows re-read the last row (their results are dropped)
  const int m = threadIdx.x & 15, kg = (threadIdx.x & 63) >> 4;
  gemm_accumulate<T, 2, NB>(w, reinterpret_cast<const T*>(a.x) + (size_t)li * Tr<T>::PARTS * kMaxCols * a.d, a.d, c.n, acc,
                            kg * R + min(m, R - 1), 4 * R);
  rstd_finish(ssp, a.d / 16, c.n, a.inv_d, a.eps, pre, s_rstd);
  if (!reduce_waves<2>(acc, dyn_red)) return;
  fold_columns<T, 2>(acc, c.n);
  const int lane = threadIdx.x & 63, col = lane & 15;
  if (col >= c.n) return;
  const float r = s_rstd[col];
  float o[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float g = acc[0][i] * r, u = acc[1][i] * r;
    o[i] = (g / (1.0f + expf(-g))) * u;
  }
  T* dst = reinterpret_cast<T*>(a.act) + (size_t)li * Tr<T>::PARTS * kMaxCols * a.F;
  const int row0 = (lane >> 4) * 4;  // of the tile
  if (R == 16) {
    store_act4<T>(dst + xoff<T>(c.n, a.F, col, t * 16 + row0), (size_t)kMaxCols * a.F, o[0], o[1], o[2], o[3]);
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int f = t * R + row0 + i;
      if (row0 + i < R && f < a.F) store_act1<T>(dst + xoff<T>(c.n, a.F, col, f), (size_t)kMaxCols * a.F, o[i]);
    }
  }
}

// ------------------------------------------------------------------------------------------
// LM head: logits + per-workgroup argmax candidates (lowest index wins ties).  grid = ceil(V/16).
// ------------------------------------------------------------------------------------------
struct HeadArgs {
  const u32x4* w;
  const void* x;  // XA slot 0: T(h * g_final)
  const float* ssp;
  float* logits;  // or null
  float* cand_val;
  int32_t* cand_idx;
  int d, V, nblk;
  float inv_d, eps;
};

__device__ __forceinline__ bool better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }

template <typename T, int NB>
__global__ __launch_bounds__(1024) void head_kernel(HeadArgs a, Cols c) {
  __shared__ float s_rstd[kMaxCols];
  const int nkt = a.d / Tr<T>::KT;
  const int t = blockIdx.x;
  const u32x4* const w[1] = {a.w + (size_t)t * nkt * 64};
  RstdPre pre;
  rstd_issue(a.ssp, a.d / 16, c.n, pre);
  f32x4 acc[1] = {{0.f, 0.f, 0.f, 0.f}};
  gemm_accumulate<T, 1, NB>(w, reinterpret_cast<const T*>(a.x), a.d, c.n, acc);
  rstd_finish(a.ssp, a.d / 16, c.n, a.inv_d, a.eps, pre, s_rstd);
  if (!reduce_waves<1>(acc, dyn_red)) return;
  fold_columns<T, 1>(acc, c.n);
  const int lane = threadIdx.x & 63, col = lane & 15;
  const bool ok = col < c.n;
  const float r = ok ? s_rstd[col] : 0.f;
  const int r0 = t * 16 + (lane >> 4) * 4;
  float bv = -INFINITY;
  int bi = 0x7FFFFFFF;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = r0 + i;
    const float v = acc[0][i] * r;
    if (ok && row < a.V) {
      if (a.logits && c.logit_row[col] >= 0) a.logits[(size_t)c.logit_row[col] * a.V + row] = v;
      if (better(v, row, bv, bi)) { bv = v; bi = row; }
    }
  }
#pragma unroll
  for (int off = 16; off <= 32; off <<= 1) {
    const float ov = __shfl_xor(bv, off, 64);
    const int oi = __shfl_xor(bi, off, 64);
    if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
  }
  if (ok && lane < 16) {
    a.cand_val[(size_t)col * a.nblk + t] = bv;
    a.cand_idx[(size_t)col * a.nblk + t] = bi;
  }
}

__global__ __launch_bounds__(1024) void argmax_final_kernel(const float* cand_val, const int32_t* cand_idx, int nblk,
                                                            int32_t* tokens_out, Cols c) {
  __shared__ float sv[16];
  __shared__ int si[16];
  const int col = blockIdx.x, tid = threadIdx.x;
  float bv = -INFINITY;
  int bi = 0x7FFFFFFF;
  for (int j0 = tid; j0 < nblk; j0 += 8 * 1024) {
    float v[8];
    int ix[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {  // independent loads, issued together
      const int j = j0 + u * 1024;
      const bool in = j < nblk;
      v[u] = in ? cand_val[(size_t)col * nblk + j] : -INFINITY;
      ix[u] = in ? cand_idx[(size_t)col * nblk + j] : 0x7FFFFFFF;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (better(v[u], ix[u], bv, bi)) { bv = v[u]; bi = ix[u]; }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float ov = __shfl_xor(bv, off, 64);
    const int oi = __shfl_xor(bi, off, 64);
    if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
  }
  if ((tid & 63) == 0) { sv[tid >> 6] = bv; si[tid >> 6] = bi; }
  __syncthreads();
  if (tid == 0) {
    for (int w = 1; w < 16; ++w)
      if (better(sv[w], si[w], bv, bi)) { bv = sv[w]; bi = si[w]; }
    if (c.out_idx[col] >= 0) tokens_out[c.out_idx[col]] = bi;
  }
}

// four consecutive elements as floats, p aligned to 4 elements
template <typename T>
__device__ __forceinline__ f32x4 load4(const T* p);
template <>
__device__ __forceinline__ f32x4 load4<float>(const float* p) {
  return *reinterpret_cast<const f32x4*>(p);
}
template <>
__device__ __forceinline__ f32x4 load4<bf16_t>(const bf16_t* p) {
  const u32x2 r = *reinterpret_cast<const u32x2*>(p);
  f32x4 v = {__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xFFFF0000u), __uint_as_float(r.y << 16),
             __uint_as_float(r.y & 0xFFFF0000u)};
  return v;
}

// ------------------------------------------------------------------------------------------
// Embedding gather: H = E[token]; sum of squares; T(H * g_attn) for the layers of the first set.
// grid = columns, 1024 threads, four elements per thread and pass.
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(1024) void embed_kernel(const T* __restrict__ E, const int32_t* __restrict__ tokens,
                                                     const float* __restrict__ gain, int n_gain, int d, int V, float* H,
                                                     T* xa, float* ssp, Cols c) {
  __shared__ float red[16];
  const int col = blockIdx.x, tid = threadIdx.x;
  const int tok = min(max(tokens[c.tok_idx[col]], 0), V - 1);  // ids outside the vocabulary are clamped
  float ss = 0.f;
  for (int j = tid * 4; j < d; j += 4096) {
    const f32x4 h = load4<T>(E + (size_t)tok * d + j);
    *reinterpret_cast<f32x4*>(H + (size_t)col * d + j) = h;
    for (int i = 0; i < n_gain; ++i) {
      const f32x4 g = *reinterpret_cast<const f32x4*>(gain + (size_t)i * d + j);
      store_act4<T>(xa + (size_t)i * Tr<T>::PARTS * kMaxCols * d + xoff<T>(c.n, d, col, j), (size_t)kMaxCols * d, h[0] * g[0], h[1] * g[1],
                    h[2] * g[2], h[3] * g[3]);
    }
    ss += (h[0] * h[0] + h[1] * h[1]) + (h[2] * h[2] + h[3] * h[3]);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
  if ((tid & 63) == 0) red[tid >> 6] = ss;
  __syncthreads();
  const int ntile = d / 16;
  float total = 0.f;
  for (int w = 0; w < 16; ++w) total += red[w];
  for (int t = tid; t < ntile; t += 1024) ssp[col * ntile + t] = (t == 0) ? total : 0.f;
}

// ------------------------------------------------------------------------------------------
// Decode attention over the KV caches of a set's layers, split along the context.
// One workgroup = (context chunk, KV head, layer x column); it serves the G query heads that
// share the KV head.  A K or V row (hd elements) is spread over LPS lanes, 16 bytes each, so a
// wave load covers SPW = 64/LPS consecutive slots (1 KB, coalesced).  Each wave walks its own
// contiguous run of slots in batches of IT loads per operand, all issued before the first is
// used, with a running (max, sum, accumulator) per query head: scores and probabilities never
// leave registers, since K and V fragments of a slot sit in the same lanes.  The four waves'
// states are combined through LDS; if the context has more than one chunk the workgroup
// writes a partial (max, sum, accumulator) per head and attn_merge_kernel combines the chunks.
// ------------------------------------------------------------------------------------------
struct AttnArgs {
  const float* Q;
  const void* kc;
  const void* vc;
  float* PO;
  float* PM;
  float* PL;
  void* AO;
  int layer0, Hq, Hkv, B, max_ctx;
  int CH;       // fixed-length cut (matrix-core kernel): slots per chunk
  int nch_ref;  // even cut (vector kernel, nb_ref > 0): chunks of a column of nb_ref batches
  int nb_ref;
  int direct;   // vector kernel: LDS holds the state of every slot group (see the kernel's last part)
  float scale;
};

// The split-KV cut of one column: its chunk count and the slot range [s0, s1) of chunk `chunk`
// (empty for chunk >= nch).  Fixed-length cut: chunks of CH slots.  Even cut: the column's
// units (of `unit` slots, the smallest step of a wave) are dealt to round(nb * nch_ref / nb_ref)
// chunks whose unit counts differ by at most one, so that a context of a power-of-two length
// plus a few drafted tokens does not leave a sliver of a chunk.
__host__ __device__ __forceinline__ void chunk_range(const AttnArgs& a, int n_slots, int unit, int chunk, int& nch, int& s0,
                                                     int& s1) {
  if (a.nb_ref == 0) {
    nch = (n_slots + a.CH - 1) / a.CH;
    s0 = chunk * a.CH;
    s1 = s0 + a.CH < n_slots ? s0 + a.CH : n_slots;
  } else {
    const int nb = (n_slots + unit - 1) / unit;
    nch = (nb * a.nch_ref + a.nb_ref / 2) / a.nb_ref;
    nch = nch > nb ? nb : nch;
    nch = nch < 1 ? 1 : nch;
    s0 = (int)((long)chunk * nb / nch) * unit;
    s1 = (int)((long)(chunk + 1) * nb / nch) * unit;
    s1 = s1 < n_slots ? s1 : n_slots;
  }
}

// The run [w0, w1) of wave `wave` of `nwv` inside the chunk [s0, s1): the chunk's units dealt evenly.
__host__ __device__ __forceinline__ void wave_range(int s0, int s1, int unit, int wave, int nwv, int& w0, int& w1) {
  const int n_units = (s1 - s0 + unit - 1) / unit;
  w0 = s0 + wave * n_units / nwv * unit;
  w1 = s0 + (wave + 1) * n_units / nwv * unit;
  w1 = w1 < s1 ? w1 : s1;
}

constexpr int kAttnIT = 8;       // loads in flight per operand per lane
constexpr int kAttnSmallIT = 2;  // the same for the short steps that finish a wave's share

// Sum over aligned groups of N lanes (8, 16 or 32), every lane of a group receiving the total,
// with data-parallel-primitive operand swizzles (lane^1 and lane^2 inside quads, then the
// mirrored lane of the other half of 8 and of 16 lanes) instead of LDS permutes.  Same operand
// pairs as an xor butterfly, hence the same bits.
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
template <int N>
__device__ __forceinline__ float group_sum(float v) {
  static_assert(N == 8 || N == 16 || N == 32, "group size");
  v += dpp_f32<0xB1>(v);   // quad_perm [1,0,3,2]
  v += dpp_f32<0x4E>(v);   // quad_perm [2,3,0,1]
  v += dpp_f32<0x141>(v);  // row_half_mirror
  if (N >= 16) v += dpp_f32<0x140>(v);  // row_mirror
  if (N >= 32) v += __shfl_xor(v, 16, 64);
  return v;
}

template <typename T, int HD>
struct AttnGeom {
  static constexpr int EPL = Tr<T>::EPL, LPS = HD / EPL, SPW = 64 / LPS;
  static constexpr int WAVE_SLOTS = kAttnIT * SPW;    // slots one wave covers per batch
  static constexpr int UNIT = kAttnSmallIT * SPW;     // and per small step: the granularity of the split
};

extern __shared__ float dyn_f[];

// TREE: the columns are nodes of token trees and carry a visibility mask; without it every
// slot up to the column's own is visible and the mask logic costs no registers.
template <typename T, int HD, int G, bool TREE>
__global__ __launch_bounds__(512) void attn_kernel(AttnArgs a, Cols c) {
  typedef AttnGeom<T, HD> Geo;
  constexpr int EPL = Geo::EPL, LPS = Geo::LPS, SPW = Geo::SPW, IT = kAttnIT;
  const int chunk = blockIdx.x, kvh = blockIdx.y;
  const int li = blockIdx.z / c.n, col = blockIdx.z % c.n;
  const int n_slots = c.pos[col] + 1;
  // slots below vis_base are all visible; slot vis_base + i (i < 64) only if bit i is set (the
  // column's row of a token tree's mask).  Causal columns have vis_base = n_slots.
  const int vbase = c.vis_base[col];
  const unsigned long long vmask = c.vis_mask[col];
  int nch, s0, s1;
  chunk_range(a, n_slots, Geo::UNIT, chunk, nch, s0, s1);
  if (chunk >= nch) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, NWV = blockDim.x >> 6;  // 4 or 8 waves
  const int sub = lane / LPS, e0 = (lane % LPS) * EPL;

  const size_t rowbase = (((size_t)(a.layer0 + li) * a.B + c.seq[col]) * a.Hkv + kvh) * (size_t)a.max_ctx;
  // wave-uniform row bases; a lane's fragment of slot s lies s * HD + e0 elements further (32-bit offsets)
  const char* kb = reinterpret_cast<const char*>(reinterpret_cast<const T*>(a.kc) + rowbase * HD);
  const char* vb = reinterpret_cast<const char*>(reinterpret_cast<const T*>(a.vc) + rowbase * HD);
  constexpr uint32_t ROW_BYTES = HD * sizeof(T);
  const uint32_t lane_byte = e0 * sizeof(T);
  const int HQ = a.Hq * HD;

  float q[G][EPL], acc[G][EPL], m_run[G], l_run[G];
  // one head per lane (see the batch code): running maximum and sum of that head only
  constexpr bool kHeadPerLane = G == 4 && LPS == 16;
  float m1 = -INFINITY, l1 = 0.f;
  const bool odd1 = lane & 1, odd2 = lane & 2;
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const float* qp = a.Q + ((size_t)li * kMaxCols + col) * HQ + (kvh * G + g) * HD + e0;
#pragma unroll
    for (int j = 0; j < EPL; ++j) {
      q[g][j] = qp[j];
      acc[g][j] = 0.f;
    }
    m_run[g] = -INFINITY;
    l_run[g] = 0.f;
  }

  // The chunk's units are dealt evenly to the waves, each taking a contiguous run [w0, w1): full
  // batches of IT loads per operand (all issued before the first is used) while more than two
  // small steps' worth is left, then small steps, so that a wave's arithmetic follows its share
  // of the slots.  Slots past w1 fetch the run's last row instead (their scores are discarded
  // below): unconditional loads, no branch per load.
  int w0, w1;
  wave_range(s0, s1, Geo::UNIT, wave, NWV, w0, w1);
  auto process = [&](auto n_loads, int base) {
    constexpr int N = decltype(n_loads)::value;
    u32x4 kr[N], vr[N];
#pragma unroll
    for (int j = 0; j < N; ++j) {
      const int s = min(base + j * SPW + sub, w1 - 1);
      kr[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kb + ((uint32_t)s * ROW_BYTES + lane_byte)));
    }
#pragma unroll
    for (int j = 0; j < N; ++j) {
      const int s = min(base + j * SPW + sub, w1 - 1);
      vr[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vb + ((uint32_t)s * ROW_BYTES + lane_byte)));
    }
    if constexpr (kHeadPerLane) {
      // Four query heads over a 16-lane row: instead of four row-wide sums per slot, the lanes
      // trade partial dot products pairwise so that lane l ends up with the row's total for head
      // 2 (l & 1) + ((l >> 1) & 1) alone; the softmax arithmetic is then done once per lane
      // (one head) and the probability of head g comes back to the row's other lanes as a
      // quad broadcast on its way into the P.V products.
      float sc1[N];
#pragma unroll
      for (int j = 0; j < N; ++j) {
        const int s = base + j * SPW + sub;
        const bool valid = s < w1 && (!TREE || s < vbase || ((vmask >> (s - vbase)) & 1ull));
        float kv[EPL];
        unpack<T>(kr[j], kv);
        float d[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          d[g] = 0.f;
#pragma unroll
          for (int e = 0; e < EPL; ++e) d[g] += q[g][e] * kv[e];
        }
        const float t0 = (odd1 ? d[2] : d[0]) + dpp_f32<0xB1>(odd1 ? d[0] : d[2]);  // lane ^ 1
        const float t1 = (odd1 ? d[3] : d[1]) + dpp_f32<0xB1>(odd1 ? d[1] : d[3]);
        float v = (odd2 ? t1 : t0) + dpp_f32<0x4E>(odd2 ? t0 : t1);                  // lane ^ 2
        v += dpp_f32<0x124>(v);  // row_ror:4
        v += dpp_f32<0x128>(v);  // row_ror:8
        sc1[j] = valid ? v * a.scale : -INFINITY;
      }
      float bm = sc1[0];
#pragma unroll
      for (int j = 1; j < N; ++j) bm = fmaxf(bm, sc1[j]);
      const float m_new = fmaxf(m1, bm);
      const float m_ref = m_new == -INFINITY ? 0.f : m_new;  // see the general path below
      const float alpha = __expf(m1 - m_ref);
      m1 = m_new;
      l1 *= alpha;
      const float al[4] = {dpp_f32<0x00>(alpha), dpp_f32<0xAA>(alpha), dpp_f32<0x55>(alpha), dpp_f32<0xFF>(alpha)};
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] *= al[g];
#pragma unroll
      for (int j = 0; j < N; ++j) {
        float vv[EPL];
        unpack<T>(vr[j], vv);
        const float p = __expf(sc1[j] - m_ref);  // 0 for slots past the end or masked
        l1 += p;
        // head g sits in quad lane 0, 2, 1, 3 for g = 0 .. 3
        const float pg[4] = {dpp_f32<0x00>(p), dpp_f32<0xAA>(p), dpp_f32<0x55>(p), dpp_f32<0xFF>(p)};
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
          for (int e = 0; e < EPL; ++e) acc[g][e] += pg[g] * vv[e];
      }
      return;
    }
    float sc[N][G], m_use[G];
#pragma unroll
    for (int j = 0; j < N; ++j) {
      const int s = base + j * SPW + sub;
      const bool valid = s < w1 && (!TREE || s < vbase || ((vmask >> (s - vbase)) & 1ull));
      float kv[EPL];
      unpack<T>(kr[j], kv);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float dot = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) dot += q[g][e] * kv[e];
        dot = group_sum<LPS>(dot);
        sc[j][g] = valid ? dot * a.scale : -INFINITY;
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float bm = sc[0][g];
#pragma unroll
      for (int j = 1; j < N; ++j) bm = fmaxf(bm, sc[j][g]);
      // The running maximum belongs to the slot group (the LPS lanes that share slots), not to the
      // wave: no cross-lane traffic per batch; the groups are brought to a common reference once,
      // after the loop.  A group whose slots so far were all past the end or masked still has
      // -inf: the exponentials then take 0 as reference and give 0 instead of exp(-inf + inf).
      const float m_new = fmaxf(m_run[g], bm);
      const float m_ref = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = __expf(m_run[g] - m_ref);  // exp(-inf) = 0 on the first batch
      m_run[g] = m_new;
      m_use[g] = m_ref;
      l_run[g] *= alpha;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] *= alpha;
    }
#pragma unroll
    for (int j = 0; j < N; ++j) {
      float vv[EPL];
      unpack<T>(vr[j], vv);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float p = __expf(sc[j][g] - m_use[g]);  // 0 for slots past the end or masked
        l_run[g] += p;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] += p * vv[e];
      }
    }
  };
  int base = w0;  // wave-uniform, like the loop conditions
  for (; w1 - base > 2 * Geo::UNIT; base += Geo::WAVE_SLOTS) process(std::integral_constant<int, IT>{}, base);
  for (; base < w1; base += Geo::UNIT) process(std::integral_constant<int, kAttnSmallIT>{}, base);

  if constexpr (kHeadPerLane) {  // back to every lane holding all four heads' maximum and sum
    const float mm[4] = {dpp_f32<0x00>(m1), dpp_f32<0xAA>(m1), dpp_f32<0x55>(m1), dpp_f32<0xFF>(m1)};
    const float ll[4] = {dpp_f32<0x00>(l1), dpp_f32<0xAA>(l1), dpp_f32<0x55>(l1), dpp_f32<0xFF>(l1)};
#pragma unroll
    for (int g = 0; g < G; ++g) {
      m_run[g] = mm[g & 3];
      l_run[g] = ll[g & 3];
    }
  }

  // Combine the NWV * SPW slot groups of the workgroup (l_run counts each slot once per group,
  // every lane of a group holds the same value).  A group, or a whole chunk of a tree column,
  // may have seen no visible slot: its maximum is -inf, its sums 0, and its weight below 0.
  const size_t arow = (size_t)li * kMaxCols + col;
  auto emit = [&](int g, int e, float m, float l, float o0, float o1) {  // outputs e, e + 1 of head g
    const int head = kvh * G + g;
    if (nch == 1) {
      T* dst = reinterpret_cast<T*>(a.AO) + (size_t)li * Tr<T>::PARTS * kMaxCols * HQ;
      store_act1<T>(dst + xoff<T>(c.n, HQ, col, head * HD + e), (size_t)kMaxCols * HQ, o0 / l);
      store_act1<T>(dst + xoff<T>(c.n, HQ, col, head * HD + e + 1), (size_t)kMaxCols * HQ, o1 / l);
    } else {
      const size_t row = arow * a.Hq + head;
      *reinterpret_cast<float2*>(a.PO + (row * kMaxChunks + chunk) * HD + e) = make_float2(o0, o1);
      if (e == 0) {
        a.PM[row * kMaxChunks + chunk] = m;
        a.PL[row * kMaxChunks + chunk] = l;
      }
    }
  };
  if (a.direct) {
    // every group's state goes to LDS as it stands; each thread then folds all groups for two
    // adjacent outputs (no cross-lane traffic at all)
    const int P = NWV * SPW, p = wave * SPW + sub;
    float* w_acc = dyn_f;              // [P][G][HD]
    float* w_m = dyn_f + P * G * HD;   // [G][P]
    float* w_l = w_m + G * P;          // [G][P]
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
      for (int e = 0; e < EPL; e += 4)
        *reinterpret_cast<f32x4*>(w_acc + (p * G + g) * HD + e0 + e) = f32x4{acc[g][e], acc[g][e + 1], acc[g][e + 2], acc[g][e + 3]};
    }
    if (lane % LPS == 0) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        w_m[g * P + p] = m_run[g];
        w_l[g * P + p] = l_run[g];
      }
    }
    __syncthreads();
    for (int idx = tid; idx < G * HD / 2; idx += blockDim.x) {
      const int g = idx / (HD / 2), e = (idx % (HD / 2)) * 2;
      float m = w_m[g * P];
      for (int q = 1; q < P; ++q) m = fmaxf(m, w_m[g * P + q]);
      const float m_ref = m == -INFINITY ? 0.f : m;
      float l = 0.f, o0 = 0.f, o1 = 0.f;
      for (int q = 0; q < P; ++q) {  // in group order: the result does not depend on timing
        const float wgt = __expf(w_m[g * P + q] - m_ref);
        const float2 v = *reinterpret_cast<const float2*>(w_acc + (q * G + g) * HD + e);
        l += w_l[g * P + q] * wgt;
        o0 += v.x * wgt;
        o1 += v.y * wgt;
      }
      emit(g, e, m, l, o0, o1);
    }
  } else {
    // LDS too small for every group: the groups of a wave are combined with shuffles first
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float mw = m_run[g];
#pragma unroll
      for (int off = LPS; off < 64; off <<= 1) mw = fmaxf(mw, __shfl_xor(mw, off, 64));
      const float rescale = m_run[g] == -INFINITY ? 0.f : __expf(m_run[g] - mw);
      m_run[g] = mw;
      l_run[g] *= rescale;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] *= rescale;
#pragma unroll
      for (int off = LPS; off < 64; off <<= 1) {
        l_run[g] += __shfl_xor(l_run[g], off, 64);
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] += __shfl_xor(acc[g][e], off, 64);
      }
    }
    float* w_acc = dyn_f;                 // [NWV][G][HD]
    float* w_m = dyn_f + NWV * G * HD;    // [NWV][G]
    float* w_l = w_m + NWV * G;           // [NWV][G]
    if (sub == 0) {
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int e = 0; e < EPL; ++e) w_acc[(wave * G + g) * HD + e0 + e] = acc[g][e];
    }
    if (lane == 0) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        w_m[wave * G + g] = m_run[g];
        w_l[wave * G + g] = l_run[g];
      }
    }
    __syncthreads();
    for (int idx = tid; idx < G * HD / 2; idx += blockDim.x) {
      const int g = idx / (HD / 2), e = (idx % (HD / 2)) * 2;
      float m = w_m[g];
      for (int w = 1; w < NWV; ++w) m = fmaxf(m, w_m[w * G + g]);
      const float m_ref = m == -INFINITY ? 0.f : m;
      float l = 0.f, o0 = 0.f, o1 = 0.f;
      for (int w = 0; w < NWV; ++w) {
        const float wgt = __expf(w_m[w * G + g] - m_ref);
        l += w_l[w * G + g] * wgt;
        o0 += w_acc[(w * G + g) * HD + e] * wgt;
        o1 += w_acc[(w * G + g) * HD + e + 1] * wgt;
      }
      emit(g, e, m, l, o0, o1);
    }
  }
}

// ------------------------------------------------------------------------------------------
// Attention on the matrix cores (bf16 caches).  The query rows that share one KV head — the G
// heads of up to 16/G columns of one sequence (the tokens of a calibration, the nodes of a tree
// level; a single column in a plain draft step) — are the 16 columns of MFMA tiles, so K and V
// are read once per group of columns and the per-slot arithmetic leaves the vector ALUs:
//   S^T[slot][row]  = K[slot][:] . Q[row][:]      A = K (rows = slots), B = Q^T, two-term bf16 q
//   O^T[e][row]    += V^T[e][slot] P^T[slot][row]  A = V^T, B = P^T, two-term bf16 p
// Each wave walks its own sub-chunk of the context in super tiles of 64 slots and leaves one
// split-KV partial per query row (merged by attn_merge_kernel; written out directly if the
// column's whole context is one sub-chunk).  The slots of a super tile are dealt to the four
// S^T tiles so that lane (row r, quarter q) ends up with the 16 CONSECUTIVE slots q*16 .. q*16+15:
// the accumulator layout of S^T is then the B-operand layout of the P.V instruction, and a
// V^T fragment is 8 consecutive slots.  V is stored [slot][head_dim]; a wave transposes its
// 64 x head_dim tile through its own piece of LDS (XOR-swizzled pieces: conflict-free 2-byte
// gathers).  grid = (ceil(sub-chunks / waves), Hkv, k * groups), block = 64 * waves.
// ------------------------------------------------------------------------------------------
struct ColGroups {
  int32_t n;                // groups
  int32_t first[kMaxCols];  // first column of group i
  int32_t count[kMaxCols];  // its columns (consecutive, same sequence); count * G <= 16
};
constexpr int kMfmaAttnWaves = 4;

__device__ __forceinline__ bf16x8 pack_bf16x8(const uint32_t (&b)[8]) {
  u32x4 v = {b[0] | (b[1] << 16), b[2] | (b[3] << 16), b[4] | (b[5] << 16), b[6] | (b[7] << 16)};
  return __builtin_bit_cast(bf16x8, v);
}

template <int HD, bool TREE>
__global__ __launch_bounds__(64 * kMfmaAttnWaves) void attn_mfma_kernel(AttnArgs a, Cols c, ColGroups cg, int G) {
  constexpr int KT = HD / 32, ET = HD / 16, PIECES = HD / 8;
  extern __shared__ u32x4 dyn_v[];  // per wave: V tile [64 slots][PIECES] then K tile [16 slots][PIECES], 16-byte pieces, swizzled
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, NWV = blockDim.x >> 6;
  const int chunk = blockIdx.x * NWV + wave, kvh = blockIdx.y;
  const int li = blockIdx.z / cg.n, grp = blockIdx.z % cg.n;
  const int first = cg.first[grp], cnt = cg.count[grp];
  const int r = lane & 15, q4 = lane >> 4;  // query row (MFMA column) and quarter / k-group
  const bool row_ok = r < cnt * G;
  const int col = first + (row_ok ? r / G : 0), g = row_ok ? r % G : 0;
  int n_max = 0;  // slots the longest column of the group attends to
  for (int i = 0; i < cnt; ++i) n_max = max(n_max, c.pos[first + i] + 1);
  const int ws0 = chunk * a.CH;
  if (ws0 >= n_max) return;  // whole wave; nothing below synchronises across waves
  const int ws1 = min(ws0 + a.CH, n_max);
  const int n_slots = c.pos[col] + 1;  // of this lane's row
  const int vbase = c.vis_base[col];
  const unsigned long long vmask = c.vis_mask[col];
  const int HQ = a.Hq * HD;
  const size_t rowbase = (((size_t)(a.layer0 + li) * a.B + c.seq[first]) * a.Hkv + kvh) * (size_t)a.max_ctx;
  const bf16_t* kc = reinterpret_cast<const bf16_t*>(a.kc) + rowbase * HD;
  const u32x4* vc = reinterpret_cast<const u32x4*>(reinterpret_cast<const bf16_t*>(a.vc) + rowbase * HD);
  u32x4* vt = dyn_v + (size_t)wave * 80 * PIECES;
  u32x4* kt_lds = vt + 64 * PIECES;
  const uint16_t* vt16 = reinterpret_cast<const uint16_t*>(vt);
  const u32x4* kc4 = reinterpret_cast<const u32x4*>(kc);

  // K and V rows of a super tile as they lie in memory (coalesced): fragment f = it*64 + lane of its
  // 64 x PIECES 16-byte pieces.  The registers are free again once their contents sit in LDS, so
  // the next super tile is requested while the current one is still being worked on; the first
  // one before the queries are fetched.
  const u32x4 zero = {0u, 0u, 0u, 0u};
  u32x4 kf[PIECES], vf[PIECES];
  auto request = [&](int base) {
#pragma unroll
    for (int it = 0; it < PIECES; ++it) {
      const int f = it * 64 + lane, sl = f / PIECES;
      kf[it] = base + sl < ws1 ? __builtin_nontemporal_load(kc4 + (size_t)base * PIECES + f) : zero;
    }
#pragma unroll
    for (int it = 0; it < PIECES; ++it) {
      const int f = it * 64 + lane, sl = f / PIECES;
      vf[it] = base + sl < ws1 ? __builtin_nontemporal_load(vc + (size_t)base * PIECES + f) : zero;
    }
  };
  request(ws0);

  // B operands of S^T: this row's query, hi and lo bf16 terms, k-group q4 of every k-tile
  bf16x8 qh[KT], ql[KT];
  {
    const float* qp = a.Q + ((size_t)li * kMaxCols + col) * HQ + (kvh * G + g) * HD + q4 * 8;
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      uint32_t hb[8], lb[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float x = row_ok ? qp[kt * 32 + e] : 0.f;
        hb[e] = float_to_bf16_bits(x);
        lb[e] = float_to_bf16_bits(x - bf16_bits_to_float(hb[e]));
      }
      qh[kt] = pack_bf16x8(hb);
      ql[kt] = pack_bf16x8(lb);
    }
  }

  f32x4 o[ET];
#pragma unroll
  for (int et = 0; et < ET; ++et) o[et] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;  // l_run: this lane's 16 slots per super tile only
  const int swz = q4 * (PIECES / 4);

  for (int base = ws0; base < ws1; base += 64) {
    // V tile into LDS with the pieces of slot s XORed by (s/16)*(PIECES/4)
#pragma unroll
    for (int it = 0; it < PIECES; ++it) {
      const int f = it * 64 + lane, sl = f / PIECES, piece = f % PIECES;
      vt[sl * PIECES + (piece ^ ((sl >> 4) * (PIECES / 4)))] = vf[it];
    }
    // scores of this lane's row against its 16 slots base + q4*16 + t*4 + i.  S^T tile t takes
    // the slots (m/4)*16 + t*4 + m%4, m = 0..15, as its A rows: their pieces go through LDS
    // (piece p of A row m stored at p ^ m, so that the 16 rows of one piece hit 16 different banks)
    float sc[4][4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
      for (int it = 0; it < PIECES; ++it) {
        const int f = it * 64 + lane, sl = f / PIECES, piece = f % PIECES;
        if (((sl >> 2) & 3) == t) {  // slot sl belongs to tile t
          const int m = (sl >> 4) * 4 + (sl & 3);
          kt_lds[m * PIECES + (piece ^ (m & (PIECES - 1)))] = kf[it];
        }
      }
      __builtin_amdgcn_wave_barrier();  // LDS operations of one wave execute in order: no wait is needed
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kt = 0; kt < KT; ++kt) {
        const u32x4 ka = kt_lds[r * PIECES + ((kt * 4 + q4) ^ (r & (PIECES - 1)))];
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka), qh[kt], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka), ql[kt], acc, 0, 0, 0);
      }
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int slot = base + q4 * 16 + t * 4 + i;
        const bool valid = row_ok && slot < n_slots && (!TREE || slot < vbase || ((vmask >> (slot - vbase)) & 1ull));
        sc[t][i] = valid ? acc[i] * a.scale : -INFINITY;
      }
    }
    if (base + 64 < ws1) request(base + 64);  // both register sets are in LDS / consumed by now
    float bm = -INFINITY;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int i = 0; i < 4; ++i) bm = fmaxf(bm, sc[t][i]);
    bm = fmaxf(bm, __shfl_xor(bm, 16, 64));  // the four quarters of a row must share the reference:
    bm = fmaxf(bm, __shfl_xor(bm, 32, 64));  // their slots are summed by one instruction below
    const float m_new = fmaxf(m_run, bm);
    const float m_ref = m_new == -INFINITY ? 0.f : m_new;  // nothing visible so far: exponentials give 0
    const float alpha = __expf(m_run - m_ref);
    m_run = m_new;
    l_run *= alpha;
#pragma unroll
    for (int et = 0; et < ET; ++et) o[et] *= alpha;
    // B operands of P.V: MFMA number h takes slots q4*16 + h*8 .. +8 of this lane = tiles 2h, 2h+1
    bf16x8 ph[2], pl[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      uint32_t hb[8], lb[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float pv = __expf(sc[2 * h + (j >> 2)][j & 3] - m_ref);
        l_run += pv;
        hb[j] = float_to_bf16_bits(pv);
        lb[j] = float_to_bf16_bits(pv - bf16_bits_to_float(hb[j]));
      }
      ph[h] = pack_bf16x8(hb);
      pl[h] = pack_bf16x8(lb);
    }
    __builtin_amdgcn_wave_barrier();
    // A operands: V^T row e = et*16 + lane%16, the 8 slots q4*16 + h*8 + j, gathered from LDS
#pragma unroll
    for (int et = 0; et < ET; ++et) {
      const int e = et * 16 + r;
      const int pofs = ((e >> 3) ^ swz) * 8 + (e & 7);  // 2-byte index inside a slot's row
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        uint32_t vb[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) vb[j] = vt16[(q4 * 16 + h * 8 + j) * HD + pofs];
        const bf16x8 va = pack_bf16x8(vb);
        o[et] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, ph[h], o[et], 0, 0, 0);
        o[et] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pl[h], o[et], 0, 0, 0);
      }
    }
    __builtin_amdgcn_wave_barrier();  // the gathers are issued before the next tile's stores into the same piece of LDS
  }

  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  if (!row_ok || ws0 >= n_slots) return;  // padding rows; columns that end before this sub-chunk
  const int nch = (n_slots + a.CH - 1) / a.CH;
  const int head = kvh * G + g;
  if (nch == 1) {
#pragma unroll
    for (int et = 0; et < ET; ++et) {
      const int e = et * 16 + q4 * 4;
      bf16_t* dst = reinterpret_cast<bf16_t*>(a.AO) + (size_t)li * 2 * kMaxCols * HQ + xoff<bf16_t>(c.n, HQ, col, head * HD + e);
      store_act4<bf16_t>(dst, (size_t)kMaxCols * HQ, o[et][0] / l_run, o[et][1] / l_run, o[et][2] / l_run, o[et][3] / l_run);
    }
  } else {
    const size_t row = ((size_t)li * kMaxCols + col) * a.Hq + head;
#pragma unroll
    for (int et = 0; et < ET; ++et)
      *reinterpret_cast<f32x4*>(a.PO + (row * kMaxChunks + chunk) * HD + et * 16 + q4 * 4) = o[et];
    if (q4 == 0) {
      a.PM[row * kMaxChunks + chunk] = m_run;
      a.PL[row * kMaxChunks + chunk] = l_run;
    }
  }
}

// Merge the chunk partials of one (layer, column, KV head): all G query heads, chunks in
// order.  Runs as its own launch: the kernel boundary is what makes the partials written by
// workgroups on other XCDs visible (a device-scope fence inside the attention kernel costs an
// L2 write-back per workgroup and was measured several times slower).  Columns whose context
// fits one chunk were finished by attn_kernel.  grid = (k * columns, Hkv), block = 256.
template <typename T, int HD>
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnArgs a, Cols c) {
  __shared__ float s_w[8][kMaxChunks];  // per head: exp(m_chunk - m) ; chunk count <= 64 = one lane each
  __shared__ float s_l[8];
  const int li = blockIdx.x / c.n, col = blockIdx.x % c.n, kvh = blockIdx.y, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int n_slots = c.pos[col] + 1;
  int nch, s0_unused, s1_unused;
  chunk_range(a, n_slots, AttnGeom<T, HD>::UNIT, 0, nch, s0_unused, s1_unused);
  if (nch == 1) return;
  const int G = a.Hq / a.Hkv, HQ = a.Hq * HD;
  const size_t arow = (size_t)li * kMaxCols + col;
  // every load of the kernel is issued up front: the first 16 chunk partials of this thread's
  // output elements (all of them for contexts up to 16 chunks) together with the chunk maxima
  // and sums, so that the kernel costs one memory latency, not three
  constexpr int EPT = (8 * HD + 255) / 256;  // output elements per thread, at most (G <= 8)
  float pv[EPT][16];
#pragma unroll
  for (int k = 0; k < EPT; ++k) {
    const int idx = tid + 256 * k;
    const int g = idx / HD, e = idx % HD;
    const float* po = a.PO + (arow * a.Hq + kvh * G + g) * kMaxChunks * HD + e;
#pragma unroll
    for (int u = 0; u < 16; ++u) pv[k][u] = (idx < G * HD && u < nch) ? po[(size_t)u * HD] : 0.f;
  }
  for (int g = wave; g < G; g += 4) {  // one wave per head, one lane per chunk
    const size_t row = arow * a.Hq + kvh * G + g;
    const float pm = lane < nch ? a.PM[row * kMaxChunks + lane] : -INFINITY;
    const float pl = lane < nch ? a.PL[row * kMaxChunks + lane] : 0.f;
    float m = pm;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    const float wgt = __expf(pm - m);
    s_w[g][lane] = wgt;
    // sum in chunk order so that the result does not depend on the reduction tree
    const float l = pl * wgt;
    float tot = 0.f;
    for (int ch = 0; ch < nch; ++ch) tot += __shfl(l, ch, 64);
    if (lane == 0) s_l[g] = tot;
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < EPT; ++k) {
    const int idx = tid + 256 * k;
    if (idx >= G * HD) break;
    const int g = idx / HD, e = idx % HD;
    const int head = kvh * G + g;
    const float* po = a.PO + (arow * a.Hq + head) * kMaxChunks * HD + e;
    float o = 0.f;
#pragma unroll
    for (int u = 0; u < 16; ++u) o += pv[k][u] * (u < nch ? s_w[g][u] : 0.f);
    for (int c0 = 16; c0 < nch; c0 += 8) {
      float pw[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) pw[u] = c0 + u < nch ? po[(size_t)(c0 + u) * HD] : 0.f;  // independent loads
#pragma unroll
      for (int u = 0; u < 8; ++u) o += pw[u] * (c0 + u < nch ? s_w[g][c0 + u] : 0.f);
    }
    store_act1<T>(reinterpret_cast<T*>(a.AO) + (size_t)li * Tr<T>::PARTS * kMaxCols * HQ + xoff<T>(c.n, HQ, col, head * HD + e),
                  (size_t)kMaxCols * HQ, o / s_l[g]);
  }
}

// ------------------------------------------------------------------------------------------
// Small utilities.
// ------------------------------------------------------------------------------------------

// Row-major [rows][K] -> tiles of R <= 16 rows, per k-tile a fragment of [k-group 4][R rows] 16-byte
// pieces (1 KB for R = 16: piece i is lane i's share of an MFMA A operand); rows padded with zeros
// up to a multiple of R.
template <typename T>
__global__ void repack_kernel(const T* __restrict__ src, u32x4* __restrict__ dst, int rows, int K, int R, size_t n_frag) {
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
  if (row < (size_t)rows) v = *reinterpret_cast<const u32x4*>(src + row * K + (size_t)kt * KT + (piece / R) * EPL);
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

// ------------------------------------------------------------------------------------------
// Launch wrappers
// ------------------------------------------------------------------------------------------

static int env_int(const char* name, int dflt) {
  const char* v = getenv(name);
  return v ? atoi(v) : dflt;
}

// Waves per workgroup (they split K).  `dflt` is the value measured best at the 8B shape for
// that operation; a wave always keeps at least 8 k-tiles.  EASYSPEC_NW_* overrides for sweeps.
static int pick_waves(int dflt, int nkt, const char* env) {
  const int forced = env_int(env, 0);
  int nw = forced > 0 ? forced : dflt;
  if (nw > 16) nw = 16;
  while (nw > 1 && nkt / nw < 8) nw /= 2;
  return nw;
}

static size_t red_bytes(int nw, int rt) { return (size_t)(nw > 1 ? nw - 1 : 0) * rt * 64 * sizeof(f32x4); }

// bf16 with more than 8 columns: hi and lo activation terms take a fragment each
static bool two_fragments(int dtype, const Cols& c) { return dtype == 1 && 2 * c.n > kMaxCols; }

#define DISPATCH_TNB(dtype, two, ...)                                         \
  do {                                                                        \
    if ((dtype) == 1 && (two)) { typedef bf16_t T; constexpr int NB = 2; __VA_ARGS__; } \
    else if ((dtype) == 1) { typedef bf16_t T; constexpr int NB = 1; __VA_ARGS__; }     \
    else { typedef float T; constexpr int NB = 1; __VA_ARGS__; }              \
  } while (0)

#define DISPATCH_T(dtype, ...)                    \
  do {                                            \
    if ((dtype) == 1) { typedef bf16_t T; __VA_ARGS__; } \
    else { typedef float T; __VA_ARGS__; }        \
  } while (0)

static size_t tile_stride(int rows, int K, int dtype, int R = 16) {  // u32x4 per matrix
  const int kt = dtype == 1 ? 32 : 16;
  return (size_t)((rows + R - 1) / R) * (K / kt) * (4 * R);
}

size_t packed_bytes(int dtype, int rows, int K, int R) { return tile_stride(rows, K, dtype, R) * sizeof(u32x4); }

// Rows per weight tile of a matrix whose launch is one workgroup per row tile.  The hardware hands
// workgroups to CUs as they free up, so a launch costs as many rounds as its busiest CU gets
// workgroups: 896 tiles of 16 rows on 256 CUs cost 4 rounds for 3.5 rounds of work.  A slightly
// lower tile (the MFMA's spare rows idle) can make the count a multiple of the CU count: 1024
// tiles of 14 rows.  More workgroups also cost more prologues and activation reads, so the tile
// is lowered only for a gain in balance of more than a tenth (measured: 14 rows at F = 14336
// take 1.5 us off a 37 us launch; 15 rows at F = 18944, balance 0.925 -> 0.987, gain nothing).
int tile_rows(int rows) {
  const int forced = env_int("EASYSPEC_TILE_ROWS", 0);  // tests: read at every create
  if (forced >= 8 && forced <= 16) return forced;
  int dev = 0, n_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1)
    n_cu = 256;
  if ((rows + 15) / 16 <= n_cu) return 16;  // less than one round anyway
  auto balance = [&](int R) {
    const int tiles = (rows + R - 1) / R;
    return (double)tiles / ((double)n_cu * ((tiles + n_cu - 1) / n_cu));
  };
  int best = 16;
  for (int R = 15; R >= 12; --R)
    if (balance(R) > balance(16) + 0.10 && balance(R) > balance(best)) best = R;
  return best;
}

void launch_repack(int dtype, const void* src, void* dst, int rows, int K, int R, hipStream_t st) {
  const size_t n_frag = tile_stride(rows, K, dtype, R);
  const unsigned grid = (unsigned)((n_frag + 255) / 256);
  DISPATCH_T(dtype, hipLaunchKernelGGL(repack_kernel<T>, dim3(grid), dim3(256), 0, st, (const T*)src, (u32x4*)dst, rows, K, R, n_frag));
}

void launch_embed(const Shape& s, const Buffers& b, const Cols& c, const int32_t* tokens, int layer0, int n_set,
                  hipStream_t st) {
  DISPATCH_T(s.dtype, hipLaunchKernelGGL(embed_kernel<T>, dim3(c.n), dim3(1024), 0, st, (const T*)b.embed, tokens,
                                         b.g_attn + (size_t)layer0 * s.d, n_set, s.d, s.V, b.H, (T*)b.XA, b.ssp, c));
}

void launch_qkv(const Shape& s, const Buffers& b, const Cols& c, int layer0, int n_set, hipStream_t st) {
  QkvArgs a;
  const size_t stride = tile_stride(s.RQKV, s.d, s.dtype);
  a.w = (const u32x4*)b.wqkv + (size_t)layer0 * stride;
  a.w_layer_stride = stride;
  a.x = b.XA;
  a.ssp = b.ssp;
  a.bias = s.has_bias ? b.bqkv + (size_t)layer0 * s.RQKV : nullptr;
  a.rope = b.rope;
  a.q = b.Q;
  a.kc = b.kc;
  a.vc = b.vc;
  a.layer0 = layer0; a.d = s.d; a.Hq = s.Hq; a.Hkv = s.Hkv; a.hd = s.hd; a.B = s.B; a.max_ctx = s.max_ctx;
  a.inv_d = 1.0f / (float)s.d; a.eps = s.eps;
  const int grid = n_set * (s.Hq + 2 * s.Hkv) * (s.hd / 32);
  const int nkt = s.d / (s.dtype == 1 ? 32 : 16);
  // few workgroups (a set of one layer): more waves per workgroup
  const int nw = pick_waves(grid < 512 ? 8 : 4, nkt, "EASYSPEC_NW_QKV");
  DISPATCH_TNB(s.dtype, two_fragments(s.dtype, c),
               hipLaunchKernelGGL((qkv_kernel<T, NB>), dim3(grid), dim3(64 * nw), red_bytes(nw, 2), st, a, c));
}

template <typename T, int HD, bool TREE>
static void launch_attn_g(int G, dim3 grid, int nwv, hipStream_t st, AttnArgs a, const Cols& c) {
  // partial state of every slot group of the workgroup if that fits the default 64 KB of
  // dynamic LDS, else of every wave
  const int groups = nwv * AttnGeom<T, HD>::SPW;
  a.direct = (size_t)groups * G * (HD + 2) * sizeof(float) <= 65536 ? 1 : 0;
  const int sets = a.direct ? groups : nwv;
  const size_t lds = (size_t)sets * G * (HD + 2) * sizeof(float);
  const dim3 blk(64 * nwv);
  switch (G) {
    case 1: hipLaunchKernelGGL((attn_kernel<T, HD, 1, TREE>), grid, blk, lds, st, a, c); break;
    case 2: hipLaunchKernelGGL((attn_kernel<T, HD, 2, TREE>), grid, blk, lds, st, a, c); break;
    case 4: hipLaunchKernelGGL((attn_kernel<T, HD, 4, TREE>), grid, blk, lds, st, a, c); break;
    case 7: hipLaunchKernelGGL((attn_kernel<T, HD, 7, TREE>), grid, blk, lds, st, a, c); break;
    case 8: hipLaunchKernelGGL((attn_kernel<T, HD, 8, TREE>), grid, blk, lds, st, a, c); break;
    default: break;  // rejected at create
  }
}

// Matrix-core attention or the vector-ALU kernel?  The MFMA kernel reads K and V once per group
// of columns of a sequence and does the per-slot arithmetic on the matrix cores, but its
// per-wave chain (LDS transposes between the two products) is longer; measured, it wins once a
// launch holds several columns of a sequence and enough (column, layer, slot) work: tree levels,
// long calibrations.  Single columns (plain draft steps) and short 1-layer launches stay on the
// vector kernel.  EASYSPEC_ATTN_MFMA = 0 / 2 forces never / always (bf16 only).
static bool attn_use_mfma(const Shape& s, const Cols& c, int n_set) {
  const int mode = env_int("EASYSPEC_ATTN_MFMA", 1);  // read at every call: tests switch it between contexts
  const long min_work = env_int("EASYSPEC_ATTN_MFMA_MIN", 30000);
  if (mode == 0 || s.dtype != 1) return false;
  if (mode == 2) return true;
  bool shared = false;
  int max_len = 1;
  for (int i = 0; i < c.n; ++i) {
    shared = shared || (i > 0 && c.seq[i] == c.seq[i - 1]);
    max_len = std::max(max_len, c.pos[i] + 1);
  }
  return shared && (long)n_set * c.n * max_len >= min_work;
}

// Runs of consecutive columns of one sequence, cut so that a group's query rows (columns x G
// heads per KV head) fill at most the 16 columns of an MFMA tile.
static void group_columns(const Cols& c, int G, ColGroups& cg) {
  const int most = std::max(1, 16 / G);
  cg.n = 0;
  for (int i = 0; i < c.n;) {
    int j = i + 1;
    while (j < c.n && c.seq[j] == c.seq[i] && j - i < most) ++j;
    cg.first[cg.n] = i;
    cg.count[cg.n] = j - i;
    ++cg.n;
    i = j;
  }
}

AttnCut attn_cut(const Shape& s, const Cols& c, int n_set) {
  AttnCut cut;
  cut.mfma = attn_use_mfma(s, c, n_set);
  cut.chunk = 0;
  cut.nb_ref = 0;
  int max_len = 1;
  for (int i = 0; i < c.n; ++i) max_len = std::max(max_len, c.pos[i] + 1);
  // Short contexts: one piece of work per (layer, column, KV head) walks the whole context, which
  // saves the merge launch; two dependent launches cost more than the narrower launch loses.
  static const int single_max = env_int("EASYSPEC_ATTN_SINGLE", 256);
  if (cut.mfma) {
    // one wave per (group of columns, sub-chunk, KV head), kMfmaAttnWaves of them per workgroup,
    // walking its sub-chunk in super tiles of 64 slots: sub-chunks of a fixed length, grown until
    // their count fits the partial buffers and the launch is not cut finer than one workgroup per CU
    // (measured: 8-wide tree level 3061 -> 2997 us against two per CU)
    ColGroups cg;
    group_columns(c, s.Hq / s.Hkv, cg);
    const int unit = 64;
    if (max_len <= single_max) {
      cut.chunk = (max_len + unit - 1) / unit * unit;
      cut.n_chunks = 1;
      return cut;
    }
    static const long max_wg = env_int("EASYSPEC_ATTN_WG", 256);
    int ch = unit;
    auto nch = [&](int ch_) { return (max_len + ch_ - 1) / ch_; };
    while (ch < 1024 && (nch(ch) > kMaxChunks || (long)nch(ch) * s.Hkv * n_set * cg.n > max_wg * kMfmaAttnWaves)) ch *= 2;
    cut.chunk = ch;
    cut.n_chunks = nch(ch);
    return cut;
  }
  return attn_cut_vector(s, c, n_set);
}

AttnCut attn_cut_vector(const Shape& s, const Cols& c, int n_set) {
  AttnCut cut;
  cut.mfma = false;
  cut.chunk = 0;
  int max_len = 1;
  for (int i = 0; i < c.n; ++i) max_len = std::max(max_len, c.pos[i] + 1);
  static const int single_max = env_int("EASYSPEC_ATTN_SINGLE", 256);
  // Vector kernel: one workgroup of four waves per (chunk, KV head, layer, column).  Every column's
  // units (the slots of a wave's small step) are dealt evenly to its chunks (chunk_range) and a
  // chunk's units evenly to its waves, which work through them in full batches of four units and
  // up to two small steps.  The chunk count of the longest column is the one that minimises the
  // arithmetic of the busiest SIMD — (workgroups per CU, rounded up) x (cost of the busiest wave
  // of a workgroup) — and among equals the smallest (fewer partials to merge).
  const int lps = s.hd * (s.dtype == 1 ? 2 : 4) / 16;
  const int unit = kAttnSmallIT * (64 / lps);
  const int nb_max = (max_len + unit - 1) / unit;
  cut.nb_ref = nb_max;
  cut.n_chunks = 1;
  if (max_len <= single_max) return cut;
  const int forced = env_int("EASYSPEC_ATTN_NCH", 0);  // tests: a fixed count for the longest column, read at every call
  static const int n_cu = [] {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
    return n;
  }();
  // cost of a wave with u units, in tenths of a full batch: a small step does a quarter of a
  // batch's slots at about a third of its time
  constexpr int per_batch = kAttnIT / kAttnSmallIT;
  auto wave_cost = [](long u) {
    const long full = u / per_batch, rest = u % per_batch;
    return 10 * full + (rest == 0 ? 0 : rest <= 2 ? 3 * rest + 1 : 10);
  };
  long best = -1;
  for (int nch = forced > 0 ? std::min(forced, nb_max) : 2; nch <= std::min(kMaxChunks, nb_max); ++nch) {
    long wgs = 0;
    for (int i = 0; i < c.n; ++i) {
      const int nb = (c.pos[i] + 1 + unit - 1) / unit;
      wgs += std::max(1, std::min(nb, (nb * nch + nb_max / 2) / nb_max));
    }
    wgs *= (long)s.Hkv * n_set;
    const long per_cu = (wgs + n_cu - 1) / n_cu;
    const long per_wave = ((nb_max + nch - 1) / nch + 3) / 4;  // units of the busiest wave
    const long score = per_cu * wave_cost(per_wave);
    if (best < 0 || score < best) {
      best = score;
      cut.n_chunks = nch;
    }
    if (forced > 0) break;
  }
  return cut;
}

int attn_waves(const AttnCut& cut) { return cut.n_chunks == 1 ? 8 : 4; }

void attn_ranges(const Shape& s, const AttnCut& cut, int n_slots, int chunk, int wave, int* nch, int* w0, int* w1) {
  AttnArgs a;
  a.CH = cut.chunk; a.nch_ref = cut.n_chunks; a.nb_ref = cut.nb_ref;
  const int lps = s.hd * (s.dtype == 1 ? 2 : 4) / 16;
  const int unit = kAttnSmallIT * (64 / lps);
  int s0, s1;
  chunk_range(a, n_slots, unit, chunk, *nch, s0, s1);
  if (chunk >= *nch) {
    *w0 = *w1 = 0;
    return;
  }
  wave_range(s0, s1, unit, wave, attn_waves(cut), *w0, *w1);
}

void launch_attn(const Shape& s, const Buffers& b, const Cols& c, int layer0, int n_set, const AttnCut& cut, hipStream_t st) {
  const int n_chunks = cut.n_chunks;
  AttnArgs a;
  a.Q = b.Q; a.kc = b.kc; a.vc = b.vc; a.PO = b.PO; a.PM = b.PM; a.PL = b.PL; a.AO = b.AO;
  a.layer0 = layer0; a.Hq = s.Hq; a.Hkv = s.Hkv; a.B = s.B; a.max_ctx = s.max_ctx;
  a.CH = cut.chunk; a.nch_ref = cut.n_chunks; a.nb_ref = cut.nb_ref;
  a.scale = 1.0f / sqrtf((float)s.hd);
  const int G = s.Hq / s.Hkv;
  const dim3 grid(n_chunks, s.Hkv, n_set * c.n);
  // one chunk per context: eight waves share the whole context of a (layer, column, KV head) and
  // no merge launch is needed; several chunks: four waves per chunk
  const int nwv = attn_waves(cut);
  bool tree = false;  // any column that does not see every slot up to its own
  for (int i = 0; i < c.n; ++i) tree = tree || c.vis_base[i] <= c.pos[i];
  if (cut.mfma) {
    ColGroups cg;
    group_columns(c, G, cg);
    const dim3 mg((n_chunks + kMfmaAttnWaves - 1) / kMfmaAttnWaves, s.Hkv, n_set * cg.n);
    const dim3 blk(64 * kMfmaAttnWaves);
    const size_t lds = (size_t)kMfmaAttnWaves * 80 * (s.hd / 8) * sizeof(u32x4);  // per wave a 64-slot V tile and a 16-slot K tile
    if (s.hd == 128 && tree) hipLaunchKernelGGL((attn_mfma_kernel<128, true>), mg, blk, lds, st, a, c, cg, G);
    else if (s.hd == 128) hipLaunchKernelGGL((attn_mfma_kernel<128, false>), mg, blk, lds, st, a, c, cg, G);
    else if (tree) hipLaunchKernelGGL((attn_mfma_kernel<64, true>), mg, blk, lds, st, a, c, cg, G);
    else hipLaunchKernelGGL((attn_mfma_kernel<64, false>), mg, blk, lds, st, a, c, cg, G);
  } else
  DISPATCH_T(s.dtype, {
    if (s.hd == 128 && tree) launch_attn_g<T, 128, true>(G, grid, nwv, st, a, c);
    else if (s.hd == 128) launch_attn_g<T, 128, false>(G, grid, nwv, st, a, c);
    else if (tree) launch_attn_g<T, 64, true>(G, grid, nwv, st, a, c);
    else launch_attn_g<T, 64, false>(G, grid, nwv, st, a, c);
  });
  if (n_chunks > 1) {
    const dim3 mgrid(n_set * c.n, s.Hkv);
    DISPATCH_T(s.dtype, {
      if (s.hd == 128) hipLaunchKernelGGL((attn_merge_kernel<T, 128>), mgrid, dim3(256), 0, st, a, c);
      else hipLaunchKernelGGL((attn_merge_kernel<T, 64>), mgrid, dim3(256), 0, st, a, c);
    });
  }
}

void launch_oproj(const Shape& s, const Buffers& b, const Cols& c, int layer0, int n_set, hipStream_t st) {
  ProjArgs a;
  const size_t stride = tile_stride(s.d, s.HQ, s.dtype);
  a.w = (const u32x4*)b.wo + (size_t)layer0 * stride;
  a.w_layer_stride = stride;
  a.x = b.AO;
  a.K = s.HQ; a.d = s.d;
  a.H = b.H; a.A = b.A; a.a_add = -1;
  a.gain = b.g_mlp + (size_t)layer0 * s.d;
  a.n_gain = 1;
  a.xout = b.XM;
  a.ssp = b.ssp;
  const int grid = n_set * (s.d / 16);
  const int nkt = s.HQ / (s.dtype == 1 ? 32 : 16);
  const int nw = pick_waves(grid < 512 ? 8 : 4, nkt, "EASYSPEC_NW_O");
  DISPATCH_TNB(s.dtype, two_fragments(s.dtype, c),
               hipLaunchKernelGGL((proj_resid_kernel<T, NB>), dim3(grid), dim3(64 * nw), red_bytes(nw, 1), st, a, c));
}

void launch_gateup(const Shape& s, const Buffers& b, const Cols& c, int layer, int n_layers, const float* ssp, hipStream_t st) {
  GateUpArgs a;
  const size_t stride = tile_stride(s.F, s.d, s.dtype, s.R_ffn);
  a.wg = (const u32x4*)b.wg + (size_t)layer * stride;
  a.wu = (const u32x4*)b.wu + (size_t)layer * stride;
  a.w_layer_stride = stride;
  a.x = b.XM; a.ssp = ssp; a.act = b.ACT; a.d = s.d; a.F = s.F; a.R = s.R_ffn;
  a.inv_d = 1.0f / (float)s.d; a.eps = s.eps;
  const int grid = n_layers * ((s.F + s.R_ffn - 1) / s.R_ffn);
  const int nkt = s.d / (s.dtype == 1 ? 32 : 16);
  const int nw = pick_waves(8, nkt, "EASYSPEC_NW_GU");
  DISPATCH_TNB(s.dtype, two_fragments(s.dtype, c),
               hipLaunchKernelGGL((gateup_kernel<T, NB>), dim3(grid), dim3(64 * nw), red_bytes(nw, 2), st, a, c));
}

void launch_down(const Shape& s, const Buffers& b, const Cols& c, int layer, int a_next, const float* gain, int n_gain,
                 void* xout, hipStream_t st) {
  ProjArgs a;
  const size_t stride = tile_stride(s.d, s.F, s.dtype);
  a.w = (const u32x4*)b.wd + (size_t)layer * stride;
  a.w_layer_stride = stride;
  a.x = b.ACT;
  a.K = s.F; a.d = s.d;
  a.H = b.H; a.A = b.A; a.a_add = a_next;
  a.gain = gain; a.n_gain = n_gain; a.xout = xout; a.ssp = b.ssp;
  const int grid = s.d / 16;
  const int nkt = s.F / (s.dtype == 1 ? 32 : 16);
  // Seven waves when that cuts K into whole batches of 8 tiles per wave (F = 14336: 8 batches each) and
  // the pass has one activation fragment: measured 11 us per step faster than eight at the 8B shape
  // (a wave's tiles are then 7 KB apart instead of a power of two); slower where K does not divide
  // (Qwen2-7B's F = 18944) or with two fragments.
  const bool seven = !two_fragments(s.dtype, c) && nkt % 56 == 0;
  const int nw = pick_waves(seven ? 7 : 8, nkt, "EASYSPEC_NW_DOWN");
  DISPATCH_TNB(s.dtype, two_fragments(s.dtype, c),
               hipLaunchKernelGGL((proj_resid_kernel<T, NB>), dim3(grid), dim3(64 * nw), red_bytes(nw, 1), st, a, c));
}

void launch_oproj_full(const Shape& s, const Buffers& b, const Cols& c, int layer0, int n_set, hipStream_t st) {
  ProjFullArgs a;
  const size_t stride = tile_stride(s.d, s.HQ, s.dtype);
  a.w = (const u32x4*)b.wo + (size_t)layer0 * stride;
  a.w_layer_stride = stride;
  a.x = b.AO;
  a.K = s.HQ; a.d = s.d; a.k = n_set; a.down = 0;
  a.H = b.H; a.A = b.A;
  a.gain = b.g_mlp + (size_t)layer0 * s.d;
  a.n_gain = 0;
  a.xout = b.XM;
  a.ssp = b.ssp_set;
  const int grid = n_set * (s.d / 16);
  const int nkt = s.HQ / (s.dtype == 1 ? 32 : 16);
  const int nw = pick_waves(grid < 512 ? 8 : 4, nkt, "EASYSPEC_NW_O");
  DISPATCH_TNB(s.dtype, two_fragments(s.dtype, c),
               hipLaunchKernelGGL((proj_full_kernel<T, NB>), dim3(grid), dim3(64 * nw), red_bytes(nw, 1), st, a, c));
}

void launch_down_full(const Shape& s, const Buffers& b, const Cols& c, int layer0, int n_set, const float* gain, int n_gain,
                      void* xout, hipStream_t st) {
  ProjFullArgs a;
  const size_t stride = tile_stride(s.d, s.F, s.dtype);
  a.w = (const u32x4*)b.wd + (size_t)layer0 * stride;
  a.w_layer_stride = stride;
  a.x = b.ACT;
  a.K = s.F; a.d = s.d; a.k = n_set; a.down = 1;
  a.H = b.H; a.A = b.A;
  a.gain = gain; a.n_gain = n_gain; a.xout = xout; a.ssp = b.ssp;
  const int grid = s.d / 16;
  const int nkt = s.F / (s.dtype == 1 ? 32 : 16);
  const int nw = pick_waves(8, nkt, "EASYSPEC_NW_DOWN");
  DISPATCH_TNB(s.dtype, two_fragments(s.dtype, c),
               hipLaunchKernelGGL((proj_full_kernel<T, NB>), dim3(grid), dim3(64 * nw), red_bytes(nw, 1), st, a, c));
}

void launch_head(const Shape& s, const Buffers& b, const Cols& c, float* logits_out, int32_t* tokens_out, hipStream_t st) {
  HeadArgs a;
  a.w = (const u32x4*)b.wlm; a.x = b.XA; a.ssp = b.ssp; a.logits = logits_out;
  a.cand_val = b.amax_val; a.cand_idx = b.amax_idx;
  a.d = s.d; a.V = s.V; a.nblk = (s.V + 15) / 16;
  a.inv_d = 1.0f / (float)s.d; a.eps = s.eps;
  const int nkt = s.d / (s.dtype == 1 ? 32 : 16);
  const int nw = pick_waves(4, nkt, "EASYSPEC_NW_HEAD");
  DISPATCH_TNB(s.dtype, two_fragments(s.dtype, c),
               hipLaunchKernelGGL((head_kernel<T, NB>), dim3(a.nblk), dim3(64 * nw), red_bytes(nw, 1), st, a, c));
  hipLaunchKernelGGL(argmax_final_kernel, dim3(c.n), dim3(1024), 0, st, a.cand_val, a.cand_idx, a.nblk, tokens_out, c);
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


