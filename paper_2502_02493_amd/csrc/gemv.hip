// Weight-streaming kernels of the EasySpec draft hot path (gfx950): QKV, O / down projection with
// the residual update, gate/up, LM head, embedding; and their launch wrappers.  The shared core
// (tile layouts, the MFMA loop, wave reduction, split RMSNorm) is in device_common.hpp.
#include "launch_common.hpp"

#include <string.h>

#include <vector>

#include "../../include/easyspec_instrument.h"

namespace es {

// ------------------------------------------------------------------------------------------
// QKV projection of the k layers of a set + bias + rotary + KV-cache write.
// The rotation pairs (row e of a head and row e + hd/2) are numbered through all heads of a layer,
// pair = head * hd/2 + e, and packed as two matrices of (Hq + 2 Hkv) * hd/2 rows each (first and
// second halves).  Unit of work: the same tile of R pairs of both, so that a pair sits in one
// lane.  R is 16, or 12 where that fills the CUs better (qkv_tile_rows); a lane's four rows stay
// inside one head because R and hd/2 are multiples of 4.  grid = k * ceil(ceil(pairs / R) / TP).
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
  int R;  // pairs per tile
  float inv_d, eps;
};

// TP: tiles of R pairs per workgroup (two where a pass loads two fragments per k-tile, as for gate/up)
// NP passes (of equal column counts) are served from one read of the weights.
template <typename T, int NB, int TP, int NP>
__device__ __forceinline__ void qkv_body(const QkvArgs* const (&ap)[NP], const Cols* const (&cp)[NP]) {
  __shared__ float s_rstd[NP][kMaxCols];
  const QkvArgs& a = *ap[0];  // what the passes share: weights, bias, rotary table, caches, shape
  const int ncols = cp[0]->n;
  const int KT = Tr<T>::KT;
  const int nkt = a.d / KT;
  const int half = a.hd / 2;
  const int R = a.R, n_pairs = (a.Hq + 2 * a.Hkv) * half, units = ceil_div(n_pairs, R), nwg = ceil_div(units, TP);
  const int li = blockIdx.x / nwg, u0 = (blockIdx.x % nwg) * TP;
  const u32x4* wl = a.w + (size_t)li * a.w_layer_stride;
  const u32x4* w[2 * TP];
#pragma unroll
  for (int p = 0; p < TP; ++p) {
    const int u = clamped_unit(u0, p, units);  // a missing last tile re-reads its neighbour (results dropped)
    w[2 * p] = wl + (size_t)u * row_tile_pieces(nkt, R);
    w[2 * p + 1] = wl + (size_t)(units + u) * row_tile_pieces(nkt, R);
  }
  // operands of the epilogue (wave 0 only) and of the norm scale are fetched before the weight
  // stream starts, so that their latency does not sit in the tail of the kernel
  const int lane = threadIdx.x & 63, col = lane & 15;
  const int row0 = (lane >> 4) * 4;  // of the tile
  const int RQKV = (a.Hq + 2 * a.Hkv) * a.hd;
  const bool col_ok = threadIdx.x < 64 && col < ncols;
  bool rows_ok[TP];
  int head[TP], e0[TP];
  f32x4 b_lo[TP], b_hi[TP];
#pragma unroll
  for (int p = 0; p < TP; ++p) {
    const int pair0 = (u0 + p) * R + row0;  // first of the lane's four pairs
    rows_ok[p] = u0 + p < units && row0 < R && pair0 < n_pairs;
    head[p] = rows_ok[p] ? pair0 / half : 0;
    e0[p] = rows_ok[p] ? pair0 % half : 0;  // element inside the head, < hd/2
    b_lo[p] = b_hi[p] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (col_ok && rows_ok[p] && a.bias) {
      b_lo[p] = *reinterpret_cast<const f32x4*>(a.bias + (size_t)li * RQKV + head[p] * a.hd + e0[p]);
      b_hi[p] = *reinterpret_cast<const f32x4*>(a.bias + (size_t)li * RQKV + head[p] * a.hd + e0[p] + half);
    }
  }
  int pos[NP], seq[NP];
  f32x4 cs01[NP][TP], cs23[NP][TP];
  const T* x[NP];
  RstdPre pre[NP];
  f32x4 acc[NP][2 * TP];
#pragma unroll
  for (int q = 0; q < NP; ++q) {
    const Cols& c = *cp[q];
    pos[q] = col_ok ? c.pos[col] : 0;
    seq[q] = col_ok ? c.seq[col] : 0;
#pragma unroll
    for (int p = 0; p < TP; ++p) {
      cs01[q][p] = cs23[q][p] = f32x4{1.f, 0.f, 1.f, 0.f};
      if (col_ok && rows_ok[p] && head[p] < a.Hq + a.Hkv) {
        const f32x4* rp = reinterpret_cast<const f32x4*>(a.rope + (size_t)c.rope_pos[col] * half + e0[p]);  // 4 x (cos, sin)
        cs01[q][p] = rp[0];
        cs23[q][p] = rp[1];
      }
    }
    x[q] = reinterpret_cast<const T*>(ap[q]->x) + (size_t)li * Tr<T>::PARTS * kMaxCols * a.d;
    rstd_issue(ap[q]->ssp, a.d / 16, ncols, pre[q]);
#pragma unroll
    for (int p = 0; p < 2 * TP; ++p) acc[q][p] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  // a tile of R < 16 pairs: the lanes of the missing rows re-read the last row (their results are dropped)
  const u32x4* const(&wc)[2 * TP] = w;
  const T* const(&xc)[NP] = x;
  gemm_accumulate<T, 2 * TP, NB, NP>(wc, xc, a.d, ncols, acc, lane_piece(lane, R), fragment_pieces(R));
  bool mine = false;
#pragma unroll
  for (int q = 0; q < NP; ++q) {
    rstd_finish(ap[q]->ssp, a.d / 16, ncols, a.inv_d, a.eps, pre[q], s_rstd[q]);
    mine = reduce_waves<2 * TP>(acc[q], red_of_pass<2 * TP>(q));
  }
  if (!mine) return;
#pragma unroll
  for (int q = 0; q < NP; ++q) fold_columns<T, 2 * TP>(acc[q], ncols);  // all 64 lanes

  if (col >= ncols) return;
#pragma unroll
  for (int q = 0; q < NP; ++q) {
    const float r = s_rstd[q][col];
#pragma unroll
    for (int p = 0; p < TP; ++p) {
      if (!rows_ok[p]) continue;
      const float cosv[4] = {cs01[q][p][0], cs01[q][p][2], cs23[q][p][0], cs23[q][p][2]},
                  sinv[4] = {cs01[q][p][1], cs01[q][p][3], cs23[q][p][1], cs23[q][p][3]};
      float lo[4], hi[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        // identity rotation (cos 1, sin 0) for the V rows; bias 0 without bias
        const float v0 = acc[q][2 * p][i] * r + b_lo[p][i], v1 = acc[q][2 * p + 1][i] * r + b_hi[p][i];
        lo[i] = v0 * cosv[i] - v1 * sinv[i];
        hi[i] = v1 * cosv[i] + v0 * sinv[i];
      }
      if (head[p] < a.Hq) {
        float* qo = ap[q]->q + ((size_t)li * kMaxCols + col) * (a.Hq * a.hd) + head[p] * a.hd + e0[p];
        store4<float>(qo, lo[0], lo[1], lo[2], lo[3]);
        store4<float>(qo + half, hi[0], hi[1], hi[2], hi[3]);
      } else {
        const bool is_k = head[p] < a.Hq + a.Hkv;
        const int kvh = is_k ? head[p] - a.Hq : head[p] - a.Hq - a.Hkv;
        T* base = reinterpret_cast<T*>(is_k ? a.kc : a.vc);
        T* row = base + ((((size_t)(a.layer0 + li) * a.B + seq[q]) * a.Hkv + kvh) * a.max_ctx + pos[q]) * a.hd + e0[p];
        store4<T>(row, lo[0], lo[1], lo[2], lo[3]);
        store4<T>(row + half, hi[0], hi[1], hi[2], hi[3]);
      }
    }
  }
}
template <typename T, int NB, int TP>
__global__ __launch_bounds__(TP == 1 ? 1024 : 512) void qkv_kernel(QkvArgs a, Cols c) {
  const QkvArgs* const ap[1] = {&a};
  const Cols* const cp[1] = {&c};
  qkv_body<T, NB, TP, 1>(ap, cp);
}
template <typename T, int NB, int TP>
__global__ __launch_bounds__(kTwinThreads) void qkv_twin_kernel(Twin<QkvArgs> t) {
  const QkvArgs* const ap[2] = {&t.a[0], &t.a[1]};
  const Cols* const cp[2] = {&t.c[0], &t.c[1]};
  qkv_body<T, NB, TP, 2>(ap, cp);
}

// ------------------------------------------------------------------------------------------
// Projection back into the residual stream: the O projections of a set's layers in one
// launch (k > 1), or one down projection (k = 1).  Layer 0 of the launch updates the
// residual: h = H + acc (+ Attnoutput of the next layer), writes H, the sum of squares of h
// and T(h * gain_j) for the consumer(s) that come next; the other layers only store their
// Attnoutput for later.  grid = k * ceil(d/16 / TP).
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

// TP: row tiles per workgroup (two for the stacked O launches of two-fragment passes, as for gate/up)
// NP passes (of equal column counts) are served from one read of the weights.
template <typename T, int NB, int TP, int NP>
__device__ __forceinline__ void proj_resid_body(const ProjArgs* const (&ap)[NP], const Cols* const (&cp)[NP]) {
  const ProjArgs& a = *ap[0];  // what the passes share: weights, gains, shape, a_add, n_gain
  const int ncols = cp[0]->n;
  const int KT = Tr<T>::KT;
  const int nkt = a.K / KT;
  const int ntile = a.d / 16, nwg = ceil_div(ntile, TP);
  const int li = blockIdx.x / nwg, t0 = (blockIdx.x % nwg) * TP;
  const u32x4* w[TP];
#pragma unroll
  for (int p = 0; p < TP; ++p)  // a missing last tile re-reads its neighbour (results dropped)
    w[p] = a.w + (size_t)li * a.w_layer_stride + (size_t)clamped_unit(t0, p, ntile) * row_tile_pieces(nkt, 16);
  // residual-update operands (wave 0 of a layer-0 workgroup) are fetched before the weight stream
  const int lane = threadIdx.x & 63, col = lane & 15;
  const bool ok = col < ncols;
  const T* x[NP];
  f32x4 h_in[NP][TP], a_in[NP][TP], g_in[TP], acc[NP][TP];
#pragma unroll
  for (int p = 0; p < TP; ++p) {
    g_in[p] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int r0 = (t0 + p) * 16 + (lane >> 4) * 4;
    if (threadIdx.x < 64 && li == 0 && ok && t0 + p < ntile) g_in[p] = *reinterpret_cast<const f32x4*>(a.gain + r0);
  }
#pragma unroll
  for (int q = 0; q < NP; ++q) {
    x[q] = reinterpret_cast<const T*>(ap[q]->x) + (size_t)li * Tr<T>::PARTS * kMaxCols * a.K;
#pragma unroll
    for (int p = 0; p < TP; ++p) {
      h_in[q][p] = a_in[q][p] = acc[q][p] = f32x4{0.f, 0.f, 0.f, 0.f};
      const int r0 = (t0 + p) * 16 + (lane >> 4) * 4;
      if (threadIdx.x < 64 && li == 0 && ok && t0 + p < ntile) {
        h_in[q][p] = *reinterpret_cast<const f32x4*>(ap[q]->H + (size_t)col * a.d + r0);
        if (a.a_add >= 0) a_in[q][p] = *reinterpret_cast<const f32x4*>(ap[q]->A + ((size_t)a.a_add * kMaxCols + col) * a.d + r0);
      }
    }
  }
  const u32x4* const(&wc)[TP] = w;
  const T* const(&xc)[NP] = x;
  gemm_accumulate<T, TP, NB, NP>(wc, xc, a.K, ncols, acc);
  bool mine = false;
#pragma unroll
  for (int q = 0; q < NP; ++q) mine = reduce_waves<TP>(acc[q], red_of_pass<TP>(q));
  if (!mine) return;
#pragma unroll
  for (int q = 0; q < NP; ++q) fold_columns<T, TP>(acc[q], ncols);  // all 64 lanes

#pragma unroll
  for (int q = 0; q < NP; ++q) {
    const ProjArgs& aq = *ap[q];
#pragma unroll
    for (int p = 0; p < TP; ++p) {
      const int t = t0 + p;
      if (t >= ntile) break;
      const int r0 = t * 16 + (lane >> 4) * 4;
      if (li > 0) {
        if (ok) store4<float>(aq.A + ((size_t)li * kMaxCols + col) * a.d + r0, acc[q][p][0], acc[q][p][1], acc[q][p][2], acc[q][p][3]);
        continue;
      }
      float ss = 0.f;
      if (ok) {
        float* hp = aq.H + (size_t)col * a.d + r0;
        f32x4 h = h_in[q][p];
        h += acc[q][p];
        if (a.a_add >= 0) h += a_in[q][p];
        *reinterpret_cast<f32x4*>(hp) = h;
        for (int j = 0; j < a.n_gain; ++j) {
          const f32x4 g = j == 0 ? g_in[p] : *reinterpret_cast<const f32x4*>(a.gain + (size_t)j * a.d + r0);
          T* xo = reinterpret_cast<T*>(aq.xout) + (size_t)j * Tr<T>::PARTS * kMaxCols * a.d + xoff<T>(ncols, a.d, col, r0);
          store_act4<T>(xo, (size_t)kMaxCols * a.d, h[0] * g[0], h[1] * g[1], h[2] * g[2], h[3] * g[3]);
        }
        ss = h[0] * h[0] + h[1] * h[1] + h[2] * h[2] + h[3] * h[3];
      }
      ss += __shfl_xor(ss, 16, 64);
      ss += __shfl_xor(ss, 32, 64);
      if (ok && lane < 16) aq.ssp[col * ntile + t] = ss;
    }
  }
}
template <typename T, int NB, int TP>
__global__ __launch_bounds__(1024) void proj_resid_kernel(ProjArgs a, Cols c) {
  const ProjArgs* const ap[1] = {&a};
  const Cols* const cp[1] = {&c};
  proj_resid_body<T, NB, TP, 1>(ap, cp);
}
template <typename T, int NB, int TP>
__global__ __launch_bounds__(kTwinThreads) void proj_resid_twin_kernel(Twin<ProjArgs> t) {
  const ProjArgs* const ap[2] = {&t.a[0], &t.a[1]};
  const Cols* const cp[2] = {&t.c[0], &t.c[1]};
  proj_resid_body<T, NB, TP, 2>(ap, cp);
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
    const u32x4* const w[1] = {a.w + (size_t)l * a.w_layer_stride + (size_t)t * row_tile_pieces(nkt, 16)};
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
// partial sums slot li and writes operand slot li of act.  grid = k * ceil(ceil(F / R) / TP).
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

// TP: row tiles of each matrix per workgroup.  Two (four MFMA row tiles share every activation
// fragment) halve the fragment loads per weight byte, which is what passes of many columns pay for.
// NP passes (of equal column counts) are served from one read of the weights.
template <typename T, int NB, int TP, int NP>
__device__ __forceinline__ void gateup_body(const GateUpArgs* const (&ap)[NP], const Cols* const (&cp)[NP]) {
  __shared__ float s_rstd[NP][kMaxCols];
  const GateUpArgs& a = *ap[0];  // what the passes share: weights and shape
  const int ncols = cp[0]->n;
  const int nkt = a.d / Tr<T>::KT;
  const int R = a.R, ntile = ceil_div(a.F, R), nunit = ceil_div(ntile, TP);
  const int li = blockIdx.x / nunit, t0 = (blockIdx.x % nunit) * TP;
  const u32x4* w[2 * TP];
#pragma unroll
  for (int p = 0; p < TP; ++p) {
    const int t = clamped_unit(t0, p, ntile);  // a missing last tile re-reads its neighbour (results dropped)
    const size_t wl = (size_t)li * a.w_layer_stride + (size_t)t * row_tile_pieces(nkt, R);
    w[2 * p] = a.wg + wl;
    w[2 * p + 1] = a.wu + wl;
  }
  const float* ssp[NP];
  const T* x[NP];
  RstdPre pre[NP];
  f32x4 acc[NP][2 * TP];
#pragma unroll
  for (int q = 0; q < NP; ++q) {
    ssp[q] = ap[q]->ssp + (size_t)li * kMaxCols * (a.d / 16);
    x[q] = reinterpret_cast<const T*>(ap[q]->x) + (size_t)li * Tr<T>::PARTS * kMaxCols * a.d;
    rstd_issue(ssp[q], a.d / 16, ncols, pre[q]);
#pragma unroll
    for (int p = 0; p < 2 * TP; ++p) acc[q][p] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  // a tile of R < 16 rows: the lanes of the missing rows re-read the last row (their results are dropped)
  const u32x4* const(&wc)[2 * TP] = w;
  const T* const(&xc)[NP] = x;
  gemm_accumulate<T, 2 * TP, NB, NP>(wc, xc, a.d, ncols, acc, lane_piece(threadIdx.x & 63, R), fragment_pieces(R));
  bool mine = false;
#pragma unroll
  for (int q = 0; q < NP; ++q) {
    rstd_finish(ssp[q], a.d / 16, ncols, a.inv_d, a.eps, pre[q], s_rstd[q]);
    mine = reduce_waves<2 * TP>(acc[q], red_of_pass<2 * TP>(q));
  }
  if (!mine) return;
#pragma unroll
  for (int q = 0; q < NP; ++q) fold_columns<T, 2 * TP>(acc[q], ncols);  // all 64 lanes
  const int lane = threadIdx.x & 63, col = lane & 15;
  if (col >= ncols) return;
  const int row0 = (lane >> 4) * 4;  // of the tile
#pragma unroll
  for (int q = 0; q < NP; ++q) {
    const float r = s_rstd[q][col];
    T* dst = reinterpret_cast<T*>(ap[q]->act) + (size_t)li * Tr<T>::PARTS * kMaxCols * a.F;
#pragma unroll
    for (int p = 0; p < TP; ++p) {
      const int t = t0 + p;
      if (t >= ntile) break;
      float o[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float g = acc[q][2 * p][i] * r, u = acc[q][2 * p + 1][i] * r;
        o[i] = (g / (1.0f + expf(-g))) * u;
      }
      if (R == 16) {
        store_act4<T>(dst + xoff<T>(ncols, a.F, col, t * 16 + row0), (size_t)kMaxCols * a.F, o[0], o[1], o[2], o[3]);
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int f = t * R + row0 + i;
          if (row0 + i < R && f < a.F) store_act1<T>(dst + xoff<T>(ncols, a.F, col, f), (size_t)kMaxCols * a.F, o[i]);
        }
      }
    }
  }
}
template <typename T, int NB, int TP>
__global__ __launch_bounds__(1024) void gateup_kernel(GateUpArgs a, Cols c) {
  const GateUpArgs* const ap[1] = {&a};
  const Cols* const cp[1] = {&c};
  gateup_body<T, NB, TP, 1>(ap, cp);
}
template <typename T, int NB, int TP>
__global__ __launch_bounds__(kTwinThreads) void gateup_twin_kernel(Twin<GateUpArgs> t) {
  const GateUpArgs* const ap[2] = {&t.a[0], &t.a[1]};
  const Cols* const cp[2] = {&t.c[0], &t.c[1]};
  gateup_body<T, NB, TP, 2>(ap, cp);
}

// ------------------------------------------------------------------------------------------
// LM head: logits + argmax candidates per row tile (lowest index wins ties).  grid = ceil(ceil(V/16) / TP).
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

// TP: row tiles per workgroup (as for gate/up: more than one where a pass loads two fragments per k-tile)
// NP passes (of equal column counts) are served from one read of the weights.
template <typename T, int NB, int TP, int NP>
__device__ __forceinline__ void head_body(const HeadArgs* const (&ap)[NP], const Cols* const (&cp)[NP]) {
  __shared__ float s_rstd[NP][kMaxCols];
  const HeadArgs& a = *ap[0];  // what the passes share: weights, shape, the logits array
  const int ncols = cp[0]->n;
  const int nkt = a.d / Tr<T>::KT;
  const int t0 = blockIdx.x * TP;
  const u32x4* w[TP];
#pragma unroll
  for (int p = 0; p < TP; ++p) w[p] = a.w + (size_t)clamped_unit(t0, p, a.nblk) * row_tile_pieces(nkt, 16);  // a missing tile re-reads the last one
  const T* x[NP];
  RstdPre pre[NP];
  f32x4 acc[NP][TP];
#pragma unroll
  for (int q = 0; q < NP; ++q) {
    x[q] = reinterpret_cast<const T*>(ap[q]->x);
    rstd_issue(ap[q]->ssp, a.d / 16, ncols, pre[q]);
#pragma unroll
    for (int p = 0; p < TP; ++p) acc[q][p] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  const u32x4* const(&wc)[TP] = w;
  const T* const(&xc)[NP] = x;
  gemm_accumulate<T, TP, NB, NP>(wc, xc, a.d, ncols, acc);
  bool mine = false;
#pragma unroll
  for (int q = 0; q < NP; ++q) {
    rstd_finish(ap[q]->ssp, a.d / 16, ncols, a.inv_d, a.eps, pre[q], s_rstd[q]);
    mine = reduce_waves<TP>(acc[q], red_of_pass<TP>(q));
  }
  if (!mine) return;
#pragma unroll
  for (int q = 0; q < NP; ++q) fold_columns<T, TP>(acc[q], ncols);  // all 64 lanes
  const int lane = threadIdx.x & 63, col = lane & 15;
  const bool ok = col < ncols;
#pragma unroll
  for (int q = 0; q < NP; ++q) {
    const HeadArgs& aq = *ap[q];
    const Cols& c = *cp[q];
    const float r = ok ? s_rstd[q][col] : 0.f;
#pragma unroll
    for (int p = 0; p < TP; ++p) {
      const int t = t0 + p;
      if (t >= a.nblk) break;
      const int r0 = t * 16 + (lane >> 4) * 4;
      float bv = -INFINITY;
      int bi = 0x7FFFFFFF;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = r0 + i;
        const float v = acc[q][p][i] * r;
        if (ok && row < a.V) {
          if (aq.logits && c.logit_row[col] >= 0) aq.logits[(size_t)c.logit_row[col] * a.V + row] = v;
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
        aq.cand_val[(size_t)col * a.nblk + t] = bv;
        aq.cand_idx[(size_t)col * a.nblk + t] = bi;
      }
    }
  }
}
template <typename T, int NB, int TP>
__global__ __launch_bounds__(1024) void head_kernel(HeadArgs a, Cols c) {
  const HeadArgs* const ap[1] = {&a};
  const Cols* const cp[1] = {&c};
  head_body<T, NB, TP, 1>(ap, cp);
}
template <typename T, int NB, int TP>
__global__ __launch_bounds__(kTwinThreads) void head_twin_kernel(Twin<HeadArgs> t) {
  const HeadArgs* const ap[2] = {&t.a[0], &t.a[1]};
  const Cols* const cp[2] = {&t.c[0], &t.c[1]};
  head_body<T, NB, TP, 2>(ap, cp);
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

// Rotation pairs per tile of the QKV matrices (16 or 12; the epilogue wants a multiple of 4).  A set
// of k layers launches k * ceil(pairs / R) workgroups; the launch costs (workgroups per CU, rounded
// up) * R rows' worth of streaming per CU.  Summed over sets of 1 to 4 layers, per layer: at the 8B
// shape (3072 pairs) tiles of 16 cost 16 + 12 + 16 + 12 (192, 384, 576, 768 workgroups on 256 CUs),
// tiles of 12 cost 12 each (256, 512, 768, 1024).
int qkv_tile_rows(int n_pairs) {
  const int forced = env_int("EASYSPEC_QKV_TILE_ROWS", 0);  // tests: read at every create
  if (forced == 8 || forced == 12 || forced == 16) return forced;
  int dev = 0, n_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1)
    n_cu = 256;
  if ((n_pairs + 15) / 16 < n_cu / 4) return 16;  // small models: never more than a fraction of a round
  auto cost = [&](int R) {
    double sum = 0.0;
    for (int k = 1; k <= 4; ++k) {
      const int wg = k * ((n_pairs + R - 1) / R);
      sum += (double)((wg + n_cu - 1) / n_cu) * R / k;
    }
    return sum;
  };
  return cost(12) < 0.9 * cost(16) ? 12 : 16;
}

void launch_embed(const Shape& s, const Buffers& b, const Cols& c, const int32_t* tokens, int layer0, int n_set,
                  hipStream_t st) {
  DISPATCH_T(s.dtype, ES_LAUNCH(embed_kernel<T>, dim3(c.n), dim3(1024), 0, st, (const T*)b.embed, tokens,
                                         b.g_attn + (size_t)layer0 * s.d, n_set, s.d, s.V, b.H, (T*)b.XA, b.ssp, c));
}

// ------------------------------------------------------------------------------------------
// Launch shapes.  One function decides, per kernel class, how a launch cuts its packed matrices into
// workgroups and waves; the launch wrappers below and the host-side walk of the weight stream
// (stream_walk) both read it from there.
// ------------------------------------------------------------------------------------------
StreamPlan stream_plan(const Shape& s, int op, int ncols, int n_layers, bool full_layer) {
  StreamPlan p;
  memset(&p, 0, sizeof p);
  p.op = op;
  p.n_layers = n_layers;
  p.R = 16;
  p.n_mat = 1;
  p.split_array = 0;
  const int kt = s.dtype == 1 ? 32 : 16;
  Cols c;
  c.n = ncols;  // the only field the choices below read
  p.NB = two_fragments(s.dtype, c) ? 2 : 1;
  int dflt_nw = 8;
  const char* env = "";
  switch (op) {
    case EASYSPEC_OP_QKV:
      p.K = s.d; p.R = s.R_qkv; p.n_mat = 2; p.split_array = 0;  // both halves in one array: first halves, then second halves
      p.units = ceil_div(s.RQKV / 2, p.R);
      p.mat_pieces = tile_stride(s.RQKV / 2, s.d, s.dtype, p.R);
      p.layer_pieces = 2 * p.mat_pieces;
      dflt_nw = n_layers * p.units < 512 ? 8 : 4;  // few workgroups (a set of one layer): more waves per workgroup
      env = "EASYSPEC_NW_QKV";
      break;
    case EASYSPEC_OP_OPROJ:
      p.K = s.HQ;
      p.units = s.d / 16;
      p.mat_pieces = p.layer_pieces = tile_stride(s.d, s.HQ, s.dtype);
      dflt_nw = n_layers * p.units < 512 ? 8 : 4;
      env = "EASYSPEC_NW_O";
      break;
    case EASYSPEC_OP_GATEUP:
      p.K = s.d; p.R = s.R_ffn; p.n_mat = 2; p.split_array = 1;  // gate and up: two arrays, same tiling
      p.units = ceil_div(s.F, p.R);
      p.mat_pieces = p.layer_pieces = tile_stride(s.F, s.d, s.dtype, p.R);
      dflt_nw = 8;
      env = "EASYSPEC_NW_GU";
      break;
    case EASYSPEC_OP_DOWN:
      p.K = s.F;
      p.units = s.d / 16;
      p.mat_pieces = p.layer_pieces = tile_stride(s.d, s.F, s.dtype);
      // Seven waves when that cuts K into whole batches of 8 tiles per wave (F = 14336: 8 batches each) and
      // the pass has one activation fragment: measured 11 us per step faster than eight at the 8B shape
      // (a wave's tiles are then 7 KB apart instead of a power of two); slower where K does not divide
      // (Qwen2-7B's F = 18944) or with two fragments.
      dflt_nw = (!full_layer && p.NB == 1 && (s.F / kt) % 56 == 0) ? 7 : 8;
      env = "EASYSPEC_NW_DOWN";
      p.n_layers = 1;  // one workgroup per row tile whatever the set size (full-layer mode sums the set's layers inside it)
      break;
    default:  // EASYSPEC_OP_HEAD
      p.K = s.d;
      p.units = (s.V + 15) / 16;
      p.mat_pieces = p.layer_pieces = tile_stride(s.V, s.d, s.dtype);
      p.n_layers = 1;
      dflt_nw = 4;
      env = "EASYSPEC_NW_HEAD";
      break;
  }
  p.nkt = p.K / kt;
  p.nw = pick_waves(dflt_nw, p.nkt, env);
  // Two units per workgroup in two-fragment passes, where the halved launch still fills the CUs (the down
  // projection's 256 workgroups never; the full-layer kernels have no such instantiation)
  p.TP = 1;
  if (op != EASYSPEC_OP_DOWN && !full_layer && pair_tiles(s.dtype, c, p.n_layers * p.units)) {
    p.TP = 2;
    if (op == EASYSPEC_OP_QKV && p.nw > 8) p.nw = 8;  // that instantiation is built for at most 8 waves
  }
  p.grid = p.n_layers * ceil_div(p.units, p.TP);
  return p;
}

// Host model of one launch: every workgroup, wave and lane computes, through the index functions the
// kernels use (tile_index.hpp), each 16-byte piece of weights and each activation fragment it would load.
int stream_walk(const Shape& s, const StreamPlan& p, int ncols, StreamWalk* r) {
  memset(r, 0, sizeof *r);
  const int EPL = s.dtype == 1 ? 8 : 4, PARTS = s.dtype == 1 ? 2 : 1;
  const int RT = p.n_mat * p.TP;       // row tiles a wave streams side by side
  const int U = batch_len(RT);
  if (U < 1) return -1;
  const int nwg = ceil_div(p.units, p.TP);
  r->w_pieces = (long long)p.n_layers * p.layer_pieces;
  r->x_slot_elems = (long long)PARTS * kOperandCols * p.K;
  r->tiles = (long long)p.n_layers * p.n_mat * p.units * p.nkt;
  std::vector<unsigned char> seen((size_t)r->tiles, 0);
  // the lanes of a wave must cover every piece of a fragment
  {
    std::vector<char> piece(fragment_pieces(p.R), 0);
    for (int lane = 0; lane < 64; ++lane) {
      const int q = lane_piece(lane, p.R);
      if (q < 0 || q >= fragment_pieces(p.R)) return -1;
      piece[q] = 1;
    }
    for (char c : piece) if (!c) ++r->uncovered_pieces;
  }
  for (int wg = 0; wg < p.grid; ++wg) {
    const int li = wg / nwg, u0 = (wg % nwg) * p.TP;
    for (int t = 0; t < p.TP; ++t) {
      const int unit = clamped_unit(u0, t, p.units);
      const bool reread = u0 + t >= p.units;
      for (int m = 0; m < p.n_mat; ++m) {
        // both halves of the QKV matrices share one array (second halves after the first); gate and up are two arrays
        const long long base = (long long)li * p.layer_pieces + (long long)((p.split_array ? 0 : m * p.units) + unit) * row_tile_pieces(p.nkt, p.R);
        for (int wave = 0; wave < p.nw; ++wave) {
          auto visit = [&](int tile) {
            for (int lane = 0; lane < 64; ++lane) {
              const long long idx = base + lane_piece(lane, p.R) + (long long)tile * fragment_pieces(p.R);
              if (idx > r->w_max) r->w_max = idx;
              if (idx < 0 || idx >= r->w_pieces) ++r->w_out_of_range;
              if (m == 0 && t == 0) {  // the activation fragments do not depend on the row tile
                for (int q = 0; q < p.NB; ++q) {
                  const long o = x_fragment_elems(EPL, PARTS, p.NB, ncols, p.K, lane, q);
                  if (o < 0) continue;
                  const long long last = o + (long long)tile * xtile_fragments(ncols) * EPL + EPL - 1;
                  if (last > r->x_max) r->x_max = last;
                  if (last >= r->x_slot_elems) ++r->x_out_of_range;
                }
              }
            }
            if (tile < 0 || tile >= p.nkt) { ++r->w_out_of_range; return; }
            if (reread) { ++r->reread_tiles; return; }
            unsigned char& n = seen[(((size_t)li * p.n_mat + m) * p.units + unit) * p.nkt + tile];
            if (n < 255) ++n;
          };
          int kt = wave;
          for (; batch_is_full(kt, U, p.nw, p.nkt); kt = next_batch(kt, U, p.nw))
            for (int u = 0; u < U; ++u) visit(batch_tile(kt, u, p.nw));
          if (kt < p.nkt)
            for (int u = 0; u < U; ++u)
              if (batch_tile(kt, u, p.nw) < p.nkt) visit(batch_tile(kt, u, p.nw));
        }
      }
    }
  }
  for (unsigned char n : seen) {
    if (n == 0) ++r->missed_tiles;
    if (n > 1) ++r->repeated_tiles;
  }
  return 0;
}

// Two passes of n_cols columns each can share their launches if no weight kernel's workgroup exceeds what the
// two-pass kernels are compiled for (twice the accumulators and activation fragments per wave).
bool twin_passes_fit(const Shape& s, int n_cols) {
  static const int ops[] = {EASYSPEC_OP_QKV, EASYSPEC_OP_OPROJ, EASYSPEC_OP_GATEUP, EASYSPEC_OP_DOWN, EASYSPEC_OP_HEAD};
  for (int op : ops)
    if (64 * stream_plan(s, op, n_cols, 1, false).nw > kTwinThreads) return false;
  return true;
}

// One pass, or (c2 given) two passes of equal column counts in one launch of the same shape, with a reduction
// buffer for each pass.
#define ES_LAUNCH_PASSES(K1, K2, grid, nw, lds, st, a, c, a2, c2)                     \
  do {                                                                                \
    if (c2) {                                                                         \
      Twin<std::decay_t<decltype(a)>> tw;                                             \
      tw.a[0] = a; tw.a[1] = a2; tw.c[0] = c; tw.c[1] = *(c2);                        \
      ES_LAUNCH(K2, dim3(grid), dim3(64 * (nw)), 2 * (lds), st, tw);                  \
    } else {                                                                          \
      ES_LAUNCH(K1, dim3(grid), dim3(64 * (nw)), lds, st, a, c);                      \
    }                                                                                 \
  } while (0)

void launch_qkv(const Shape& s, const Buffers& b, const Cols& c, int layer0, int n_set, hipStream_t st, const Buffers* b2,
                const Cols* c2) {
  const StreamPlan p = stream_plan(s, EASYSPEC_OP_QKV, c.n, n_set, false);
  auto args = [&](const Buffers& w) {
    QkvArgs a;
    a.w = (const u32x4*)w.wqkv + (size_t)layer0 * p.layer_pieces;
    a.w_layer_stride = p.layer_pieces;
    a.x = w.XA;
    a.ssp = w.ssp;
    a.bias = s.has_bias ? w.bqkv + (size_t)layer0 * s.RQKV : nullptr;
    a.rope = w.rope;
    a.q = w.Q;
    a.kc = w.kc;
    a.vc = w.vc;
    a.layer0 = layer0; a.d = s.d; a.Hq = s.Hq; a.Hkv = s.Hkv; a.hd = s.hd; a.B = s.B; a.max_ctx = s.max_ctx;
    a.R = p.R;
    a.inv_d = 1.0f / (float)s.d; a.eps = s.eps;
    return a;
  };
  const QkvArgs a = args(b), a2 = args(b2 ? *b2 : b);
  if (p.TP == 2) {
    // two tiles per workgroup share every fragment load (12-wide tree level 3292 -> 3282 us)
    ES_LAUNCH_PASSES((qkv_kernel<bf16_t, 2, 2>), (qkv_twin_kernel<bf16_t, 2, 2>), p.grid, p.nw, red_bytes(p.nw, 4), st, a, c, a2, c2);
    return;
  }
  DISPATCH_TNB(s.dtype, p.NB == 2,
               ES_LAUNCH_PASSES((qkv_kernel<T, NB, 1>), (qkv_twin_kernel<T, NB, 1>), p.grid, p.nw, red_bytes(p.nw, 2), st, a, c, a2, c2));
}

void launch_oproj(const Shape& s, const Buffers& b, const Cols& c, int layer0, int n_set, hipStream_t st, const Buffers* b2,
                  const Cols* c2) {
  const StreamPlan p = stream_plan(s, EASYSPEC_OP_OPROJ, c.n, n_set, false);
  auto args = [&](const Buffers& w) {
    ProjArgs a;
    a.w = (const u32x4*)w.wo + (size_t)layer0 * p.layer_pieces;
    a.w_layer_stride = p.layer_pieces;
    a.x = w.AO;
    a.K = s.HQ; a.d = s.d;
    a.H = w.H; a.A = w.A; a.a_add = -1;
    a.gain = w.g_mlp + (size_t)layer0 * s.d;
    a.n_gain = 1;
    a.xout = w.XM;
    a.ssp = w.ssp;
    return a;
  };
  const ProjArgs a = args(b), a2 = args(b2 ? *b2 : b);
  if (p.TP == 2) {
    // two row tiles per workgroup share every fragment load (12-wide tree level 3284 -> 3259 us)
    ES_LAUNCH_PASSES((proj_resid_kernel<bf16_t, 2, 2>), (proj_resid_twin_kernel<bf16_t, 2, 2>), p.grid, p.nw, red_bytes(p.nw, 2), st, a, c, a2, c2);
    return;
  }
  DISPATCH_TNB(s.dtype, p.NB == 2,
               ES_LAUNCH_PASSES((proj_resid_kernel<T, NB, 1>), (proj_resid_twin_kernel<T, NB, 1>), p.grid, p.nw, red_bytes(p.nw, 1), st, a, c, a2, c2));
}

void launch_gateup(const Shape& s, const Buffers& b, const Cols& c, int layer, int n_layers, const float* ssp, hipStream_t st,
                   const Buffers* b2, const Cols* c2, const float* ssp2) {
  const StreamPlan p = stream_plan(s, EASYSPEC_OP_GATEUP, c.n, n_layers, false);
  auto args = [&](const Buffers& w, const float* sums) {
    GateUpArgs a;
    a.wg = (const u32x4*)w.wg + (size_t)layer * p.layer_pieces;
    a.wu = (const u32x4*)w.wu + (size_t)layer * p.layer_pieces;
    a.w_layer_stride = p.layer_pieces;
    a.x = w.XM; a.ssp = sums; a.act = w.ACT; a.d = s.d; a.F = s.F; a.R = p.R;
    a.inv_d = 1.0f / (float)s.d; a.eps = s.eps;
    return a;
  };
  const GateUpArgs a = args(b, ssp), a2 = args(b2 ? *b2 : b, b2 ? ssp2 : ssp);
  if (p.TP == 2) {
    // two fragments per k-tile: two row tiles of each matrix per workgroup, so that four MFMA row tiles
    // share every fragment load (measured: 12-wide tree level 3402 -> 3322 us; with one fragment the
    // larger workgroups lose: 6-token calibration 3377 -> 3411 us, draft step 2676 -> 2731 us)
    ES_LAUNCH_PASSES((gateup_kernel<bf16_t, 2, 2>), (gateup_twin_kernel<bf16_t, 2, 2>), p.grid, p.nw, red_bytes(p.nw, 4), st, a, c, a2, c2);
    return;
  }
  DISPATCH_TNB(s.dtype, p.NB == 2,
               ES_LAUNCH_PASSES((gateup_kernel<T, NB, 1>), (gateup_twin_kernel<T, NB, 1>), p.grid, p.nw, red_bytes(p.nw, 2), st, a, c, a2, c2));
}

void launch_down(const Shape& s, const Buffers& b, const Cols& c, int layer, int a_next, const float* gain, int n_gain,
                 void* xout, hipStream_t st, const Buffers* b2, const Cols* c2, void* xout2) {
  const StreamPlan p = stream_plan(s, EASYSPEC_OP_DOWN, c.n, 1, false);
  auto args = [&](const Buffers& w, void* out) {
    ProjArgs a;
    a.w = (const u32x4*)w.wd + (size_t)layer * p.layer_pieces;
    a.w_layer_stride = p.layer_pieces;
    a.x = w.ACT;
    a.K = s.F; a.d = s.d;
    a.H = w.H; a.A = w.A; a.a_add = a_next;
    a.gain = gain; a.n_gain = n_gain; a.xout = out; a.ssp = w.ssp;
    return a;
  };
  const ProjArgs a = args(b, xout), a2 = args(b2 ? *b2 : b, b2 ? xout2 : xout);
  DISPATCH_TNB(s.dtype, p.NB == 2,
               ES_LAUNCH_PASSES((proj_resid_kernel<T, NB, 1>), (proj_resid_twin_kernel<T, NB, 1>), p.grid, p.nw, red_bytes(p.nw, 1), st, a, c, a2, c2));
}

void launch_oproj_full(const Shape& s, const Buffers& b, const Cols& c, int layer0, int n_set, hipStream_t st) {
  ProjFullArgs a;
  const StreamPlan p = stream_plan(s, EASYSPEC_OP_OPROJ, c.n, n_set, true);
  a.w = (const u32x4*)b.wo + (size_t)layer0 * p.layer_pieces;
  a.w_layer_stride = p.layer_pieces;
  a.x = b.AO;
  a.K = s.HQ; a.d = s.d; a.k = n_set; a.down = 0;
  a.H = b.H; a.A = b.A;
  a.gain = b.g_mlp + (size_t)layer0 * s.d;
  a.n_gain = 0;
  a.xout = b.XM;
  a.ssp = b.ssp_set;
  DISPATCH_TNB(s.dtype, p.NB == 2,
               ES_LAUNCH((proj_full_kernel<T, NB>), dim3(p.grid), dim3(64 * p.nw), red_bytes(p.nw, 1), st, a, c));
}

void launch_down_full(const Shape& s, const Buffers& b, const Cols& c, int layer0, int n_set, const float* gain, int n_gain,
                      void* xout, hipStream_t st) {
  ProjFullArgs a;
  const StreamPlan p = stream_plan(s, EASYSPEC_OP_DOWN, c.n, n_set, true);
  a.w = (const u32x4*)b.wd + (size_t)layer0 * p.layer_pieces;
  a.w_layer_stride = p.layer_pieces;
  a.x = b.ACT;
  a.K = s.F; a.d = s.d; a.k = n_set; a.down = 1;
  a.H = b.H; a.A = b.A;
  a.gain = gain; a.n_gain = n_gain; a.xout = xout; a.ssp = b.ssp;
  DISPATCH_TNB(s.dtype, p.NB == 2,
               ES_LAUNCH((proj_full_kernel<T, NB>), dim3(p.grid), dim3(64 * p.nw), red_bytes(p.nw, 1), st, a, c));
}

void launch_head(const Shape& s, const Buffers& b, const Cols& c, float* logits_out, int32_t* tokens_out, hipStream_t st,
                 const Buffers* b2, const Cols* c2) {
  const StreamPlan p = stream_plan(s, EASYSPEC_OP_HEAD, c.n, 1, false);
  auto args = [&](const Buffers& w) {
    HeadArgs a;
    a.w = (const u32x4*)w.wlm; a.x = w.XA; a.ssp = w.ssp; a.logits = logits_out;
    a.cand_val = w.amax_val; a.cand_idx = w.amax_idx;
    a.d = s.d; a.V = s.V; a.nblk = p.units;
    a.inv_d = 1.0f / (float)s.d; a.eps = s.eps;
    return a;
  };
  const HeadArgs a = args(b), a2 = args(b2 ? *b2 : b);
  if (p.TP == 2) {
    // two row tiles per workgroup share every fragment load (12-wide tree level 3309 -> 3276 us; four: the same)
    ES_LAUNCH_PASSES((head_kernel<bf16_t, 2, 2>), (head_twin_kernel<bf16_t, 2, 2>), p.grid, p.nw, red_bytes(p.nw, 2), st, a, c, a2, c2);
  } else {
    DISPATCH_TNB(s.dtype, p.NB == 2,
                 ES_LAUNCH_PASSES((head_kernel<T, NB, 1>), (head_twin_kernel<T, NB, 1>), p.grid, p.nw, red_bytes(p.nw, 1), st, a, c, a2, c2));
  }
  ES_LAUNCH(argmax_final_kernel, dim3(c.n), dim3(1024), 0, st, a.cand_val, a.cand_idx, a.nblk, tokens_out, c);
  if (c2) ES_LAUNCH(argmax_final_kernel, dim3(c2->n), dim3(1024), 0, st, a2.cand_val, a2.cand_idx, a2.nblk, tokens_out, *c2);
}

}  // namespace es
