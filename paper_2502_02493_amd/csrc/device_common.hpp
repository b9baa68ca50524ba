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
#pragma once
#include "kernels.h"
#include "tile_index.hpp"

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

// Layout of an activation operand: see tile_index.hpp (xoff_elems), here by element type.
static_assert(kOperandCols == kMaxCols, "operand slots hold kMaxCols columns");
template <typename T>
__device__ __forceinline__ size_t xoff(int ncols, int K, int col, int k) {
  return xoff_elems(Tr<T>::EPL, ncols, K, col, k);
}
// u32x4 between the fragments of consecutive k-tiles
template <typename T>
__device__ __forceinline__ int xtile_stride(int ncols) {
  return xtile_fragments(ncols);
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ uint32_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);  // round to nearest, ties to even
  return u >> 16;
}

// two floats to two bf16 (a in the low half), round to nearest even: one v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
// x[0..7] as two bf16 terms, hi = bf16(x), lo = bf16(x - hi)
__device__ __forceinline__ void split_bf16x8(const float (&x)[8], bf16x8& hi, bf16x8& lo) {
  uint32_t h[4], l[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    h[j] = pack_bf16x2(x[2 * j], x[2 * j + 1]);
    l[j] = pack_bf16x2(x[2 * j] - __uint_as_float(h[j] << 16), x[2 * j + 1] - __uint_as_float(h[j] & 0xFFFF0000u));
  }
  const u32x4 hv = {h[0], h[1], h[2], h[3]}, lv = {l[0], l[1], l[2], l[3]};
  hi = __builtin_bit_cast(bf16x8, hv);
  lo = __builtin_bit_cast(bf16x8, lv);
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

// NP = forward passes served by one launch (1, or 2: a calibration of more columns than one pass holds runs
// its passes two at a time).  Every weight fragment a wave loads is then used for both passes' columns: the
// passes have their own activation operands, accumulators and epilogues, the weights leave HBM once.
template <typename T, int RT, int NB, int NP>
__device__ __forceinline__ void gemm_loop(const u32x4* const (&w)[RT], const u32x4* const (&xp)[NP][NB], int xs, bool colok,
                                          int nkt, f32x4 (&acc)[NP][RT], int w_lane, int w_stride) {
  constexpr int U = batch_len(RT);  // k-tiles per batch: 8 KB of weights in flight per wave
  const int wave = threadIdx.x >> 6, NW = blockDim.x >> 6;
  // w_lane: the lane's 16-byte piece of a weight fragment, w_stride: pieces per fragment (lane and 64 for tiles of 16 rows)
  const u32x4* wp[RT];
#pragma unroll
  for (int r = 0; r < RT; ++r) wp[r] = w[r] + w_lane;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  int kt = wave;
  for (; batch_is_full(kt, U, NW, nkt); kt = next_batch(kt, U, NW)) {
    u32x4 a[RT][U], b[NP][NB][U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int r = 0; r < RT; ++r) a[r][u] = __builtin_nontemporal_load(wp[r] + (size_t)batch_tile(kt, u, NW) * w_stride);
    }
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
      for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int q = 0; q < NB; ++q) b[p][q][u] = colok ? xp[p][q][(size_t)batch_tile(kt, u, NW) * xs] : zero;
      }
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int r = 0; r < RT; ++r) {
#pragma unroll
        for (int p = 0; p < NP; ++p)
#pragma unroll
          for (int q = 0; q < NB; ++q) mma<T>(acc[p][r], a[r][u], b[p][q][u]);
      }
    }
  }
  if (kt < nkt) {
    // last, partial batch: same shape with the loads past the end switched off (wave-uniform), so
    // that the remaining tiles are still fetched together instead of one latency at a time
    u32x4 a[RT][U], b[NP][NB][U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool in = batch_tile(kt, u, NW) < nkt;
#pragma unroll
      for (int r = 0; r < RT; ++r) a[r][u] = in ? __builtin_nontemporal_load(wp[r] + (size_t)batch_tile(kt, u, NW) * w_stride) : zero;
    }
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const bool in = colok && batch_tile(kt, u, NW) < nkt;
#pragma unroll
        for (int q = 0; q < NB; ++q) b[p][q][u] = in ? xp[p][q][(size_t)batch_tile(kt, u, NW) * xs] : zero;
      }
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int r = 0; r < RT; ++r) {
#pragma unroll
        for (int p = 0; p < NP; ++p)
#pragma unroll
          for (int q = 0; q < NB; ++q) mma<T>(acc[p][r], a[r][u], b[p][q][u]);
      }
    }
  }
}

// NB is chosen by the host per launch: 1 when the activations have one term (fp32) or the
// columns fold (at most 8), else 2.  Separate instantiations keep the common one-fragment path
// free of the second path's registers.  x[p]: the operand of pass p (all passes have ncols columns).
template <typename T, int RT, int NB, int NP>
__device__ __forceinline__ void gemm_accumulate(const u32x4* const (&w)[RT], const T* const (&x)[NP], int K, int ncols,
                                                f32x4 (&acc)[NP][RT], int w_lane = -1, int w_stride = 64) {
  constexpr int EPL = Tr<T>::EPL, KT = Tr<T>::KT, PARTS = Tr<T>::PARTS;
  const int lane = threadIdx.x & 63;
  const int nkt = K / KT;
  if (w_lane < 0) w_lane = lane;  // full tiles: fragment piece i belongs to lane i
  // NB == 1: lane column c < ncols reads the hi term of column c, column ncols + c its lo term
  long o[NB];
#pragma unroll
  for (int q = 0; q < NB; ++q) o[q] = x_fragment_elems(EPL, PARTS, NB, ncols, K, lane, q);
  const bool colok = o[0] >= 0;
  const u32x4* xp[NP][NB];
#pragma unroll
  for (int p = 0; p < NP; ++p)
#pragma unroll
    for (int q = 0; q < NB; ++q) xp[p][q] = reinterpret_cast<const u32x4*>(x[p] + (colok ? o[q] : 0));
  const u32x4* const(&xc)[NP][NB] = xp;
  gemm_loop<T, RT, NB, NP>(w, xc, xtile_stride<T>(ncols), colok, nkt, acc, w_lane, w_stride);
}

// one pass
template <typename T, int RT, int NB>
__device__ __forceinline__ void gemm_accumulate(const u32x4* const (&w)[RT], const T* __restrict__ x, int K, int ncols,
                                                f32x4 (&acc)[RT], int w_lane = -1, int w_stride = 64) {
  const T* const xs[1] = {x};
  gemm_accumulate<T, RT, NB, 1>(w, xs, K, ncols, reinterpret_cast<f32x4(&)[1][RT]>(acc), w_lane, w_stride);
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

// Kernel argument of a launch that serves two passes: their arguments and columns side by side.  Those kernels
// are compiled for workgroups of at most kTwinThreads threads (room for 256 registers per lane).
constexpr int kTwinThreads = 512;
template <typename Args>
struct Twin {
  Args a[2];
  Cols c[2];
};
// pass p's piece of the reduction buffer ((NW - 1) * RT * 64 f32x4 each)
template <int RT>
__device__ __forceinline__ f32x4* red_of_pass(int p) {
  const int NW = blockDim.x >> 6;
  return dyn_red + (size_t)p * (NW > 1 ? NW - 1 : 0) * RT * 64;
}

}  // namespace es
