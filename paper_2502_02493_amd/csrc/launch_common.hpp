// Host-side helpers shared by the launch wrappers of the kernel files.
#pragma once
#include "device_common.hpp"

#include <hip/hip_ext.h>
#include <stdlib.h>

namespace es {

static inline int env_int(const char* name, int dflt) {
  const char* v = getenv(name);
  return v ? atoi(v) : dflt;
}

// Waves per workgroup (they split K).  `dflt` is the value measured best at the 8B shape for
// that operation; a wave always keeps at least 8 k-tiles.  EASYSPEC_NW_* overrides for sweeps.
static inline int pick_waves(int dflt, int nkt, const char* env) {
  const int forced = env_int(env, 0);
  int nw = forced > 0 ? forced : dflt;
  if (nw > 16) nw = 16;
  while (nw > 1 && nkt / nw < 8) nw /= 2;
  return nw;
}

// Every launch of the forward pass goes through here; see LaunchTimer.
#define ES_LAUNCH(kernel, grid, block, lds, st, ...)                                                              \
  do {                                                                                                            \
    es::LaunchTimer* t_ = es::g_launch_timer;                                                                     \
    if (t_ && t_->used + 2 <= t_->cap) {                                                                          \
      hipExtLaunchKernelGGL(kernel, grid, block, lds, st, t_->ev[t_->used], t_->ev[t_->used + 1], 0, __VA_ARGS__); \
      t_->op[t_->used / 2] = (int8_t)t_->cur_op;                                                                  \
      t_->used += 2;                                                                                              \
    } else {                                                                                                      \
      hipLaunchKernelGGL(kernel, grid, block, lds, st, __VA_ARGS__);                                              \
    }                                                                                                             \
  } while (0)

static inline size_t red_bytes(int nw, int rt) { return (size_t)(nw > 1 ? nw - 1 : 0) * rt * 64 * sizeof(f32x4); }

// bf16 with more than 8 columns: hi and lo activation terms take a fragment each
static inline bool two_fragments(int dtype, const Cols& c) { return dtype == 1 && 2 * c.n > kMaxCols; }

static inline int cu_count() {
  static const int n_cu = [] {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
    return n;
  }();
  return n_cu;
}

// Two-fragment passes: may the workgroups of a launch of n one-tile workgroups take two row tiles each
// (every activation fragment load then serves twice the weights)?  Only where the halved launch does
// not cost the busiest CU more tiles than before: 1024 -> 512 workgroups on 256 CUs stays at four
// tiles per CU, 768 -> 384 would go from three to four (Qwen2-7B shape, 12-wide tree level: 3407 us
// without pairing, 3434 us with every launch paired).
static inline bool pair_tiles(int dtype, const Cols& c, int n) {
  if (!two_fragments(dtype, c)) return false;
  const int forced = env_int("EASYSPEC_PAIR_TILES", -1);  // tests (small models never fill a round): read at every call
  if (forced >= 0) return forced != 0;
  const int n_cu = cu_count();
  return 2 * (((n + 1) / 2 + n_cu - 1) / n_cu) <= (n + n_cu - 1) / n_cu;
}

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

static inline size_t tile_stride(int rows, int K, int dtype, int R = 16) {  // u32x4 per matrix
  const int kt = dtype == 1 ? 32 : 16;
  return (size_t)((rows + R - 1) / R) * (K / kt) * (4 * R);
}

}  // namespace es
