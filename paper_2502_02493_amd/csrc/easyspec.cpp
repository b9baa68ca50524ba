// Host side of the EasySpec C ABI (include/easyspec.h): argument checks, the per-sequence
// precise / fuzzy length state machine, weight repacking, and the launch sequence of one
// forward pass.  All arithmetic of the method runs in the kernels of gemv.hip, attention.hip and accept.hip.
#include "../../include/easyspec.h"
#include "../../include/easyspec_instrument.h"

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <string>
#include <vector>

#include "kernels.h"
#include "tile_index.hpp"

using namespace es;

struct easyspec_ctx {
  easyspec_config cfg;
  Shape s;
  Buffers b;
  Buffers b2;      // a second set of per-pass workspaces (same weights and caches): the second of two passes run together
  bool has_b2;
  const float* last_H;  // residual rows of the most recent pass
  hipStream_t stream;
  bool weights_loaded;
  std::vector<int32_t> precise, fuzzy;
  // token tree of each sequence (nodes = its fuzzy slots, node t in slot precise + t)
  struct Tree {
    int32_t n = 0;
    int32_t depth[EASYSPEC_MAX_TREE_NODES];
    uint64_t line[EASYSPEC_MAX_TREE_NODES];  // bit a set: node a is the node itself or an ancestor
  };
  std::vector<Tree> tree;
  std::vector<int32_t> bounds;  // current layer-parallel strategy
  std::vector<int32_t> single;  // every layer alone (Alg. 1 order)
  std::vector<void*> allocs;
  std::vector<std::pair<void*, size_t>> work;  // the per-pass workspaces (easyspec_poison_workspaces)
  int32_t last_rows;
  int32_t parallel_mode;  // EASYSPEC_PARALLEL_*
  // per-kernel timing (easyspec_profile_*)
  int32_t prof_op;
  std::vector<hipEvent_t> prof_ev;  // start/stop pairs
  std::vector<int8_t> prof_op_of;   // kernel class of the launch that took pair i
  LaunchTimer timer;                // the pairs handed to the launches of the profiled kernel class
  std::string err;
};

static thread_local std::string g_err;
thread_local es::LaunchTimer* es::g_launch_timer = nullptr;

static int fail(easyspec_ctx* ctx, int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (ctx) ctx->err = buf;
  else g_err = buf;
  return code;
}

#define HIPCHK(ctx, call)                                                                           \
  do {                                                                                              \
    hipError_t e_ = (call);                                                                         \
    if (e_ != hipSuccess) return fail(ctx, EASYSPEC_EHIP, "%s: %s", #call, hipGetErrorString(e_)); \
  } while (0)

static size_t esize(const Shape& s) { return s.dtype == EASYSPEC_DTYPE_BF16 ? 2 : 4; }
static size_t packed_bytes(const Shape& s, int rows, int K, int R = 16) { return es::packed_bytes(s.dtype, rows, K, R); }

static int dev_alloc(easyspec_ctx* ctx, void** p, size_t bytes) {
  *p = nullptr;
  if (bytes == 0) bytes = 16;
  HIPCHK(ctx, hipMalloc(p, bytes));
  ctx->allocs.push_back(*p);
  return EASYSPEC_OK;
}

#define ALLOC(ctx, ptr, bytes)                                       \
  do {                                                               \
    int rc_ = dev_alloc(ctx, (void**)&(ptr), (size_t)(bytes));       \
    if (rc_ != EASYSPEC_OK) return rc_;                              \
  } while (0)
// a workspace that every forward pass writes before it reads it
#define ALLOC_WORK(ctx, ptr, bytes)                                  \
  do {                                                               \
    ALLOC(ctx, ptr, bytes);                                          \
    (ctx)->work.emplace_back((void*)(ptr), (size_t)(bytes));         \
  } while (0)

static int check_config(const easyspec_config* c) {
  if (!c) return fail(nullptr, EASYSPEC_EINVAL, "config is NULL");
  if (c->n_layers < 1 || c->d_model < 32 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->d_ffn < 32 || c->vocab < 1)
    return fail(nullptr, EASYSPEC_EINVAL, "non-positive model dimension");
  if (c->dtype != EASYSPEC_DTYPE_F32 && c->dtype != EASYSPEC_DTYPE_BF16) return fail(nullptr, EASYSPEC_EINVAL, "unknown dtype %d", c->dtype);
  if (c->head_dim != 64 && c->head_dim != 128) return fail(nullptr, EASYSPEC_EINVAL, "head_dim must be 64 or 128, got %d", c->head_dim);
  if (c->d_model % 32 || c->d_ffn % 32 || (c->n_q_heads * c->head_dim) % 32)
    return fail(nullptr, EASYSPEC_EINVAL, "d_model, d_ffn and n_q_heads*head_dim must be multiples of 32");
  if (c->n_q_heads % c->n_kv_heads) return fail(nullptr, EASYSPEC_EINVAL, "n_q_heads must be a multiple of n_kv_heads");
  const int g = c->n_q_heads / c->n_kv_heads;
  if (g != 1 && g != 2 && g != 4 && g != 7 && g != 8)
    return fail(nullptr, EASYSPEC_EINVAL, "n_q_heads/n_kv_heads = %d is not one of 1, 2, 4, 7, 8", g);
  if (c->max_batch < 1 || c->max_batch > EASYSPEC_MAX_BATCH) return fail(nullptr, EASYSPEC_EINVAL, "max_batch must be 1..%d", EASYSPEC_MAX_BATCH);
  if (c->max_calib_tokens < 1 || c->max_calib_tokens > EASYSPEC_MAX_CALIB_TOKENS)
    return fail(nullptr, EASYSPEC_EINVAL, "max_calib_tokens must be 1..%d", EASYSPEC_MAX_CALIB_TOKENS);
  if (c->max_ctx < 1 || c->max_ctx > kMaxChunks * 1024) return fail(nullptr, EASYSPEC_EINVAL, "max_ctx must be 1..%d", kMaxChunks * 1024);
  if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f)) return fail(nullptr, EASYSPEC_EINVAL, "bad rms_eps or rope_theta");
  return EASYSPEC_OK;
}

static void shape_of(const easyspec_config* cfg, Shape& s) {
  memset(&s, 0, sizeof s);
  s.dtype = cfg->dtype; s.L = cfg->n_layers; s.d = cfg->d_model; s.Hq = cfg->n_q_heads; s.Hkv = cfg->n_kv_heads;
  s.hd = cfg->head_dim; s.F = cfg->d_ffn; s.V = cfg->vocab; s.HQ = s.Hq * s.hd; s.RQKV = (s.Hq + 2 * s.Hkv) * s.hd;
  s.B = cfg->max_batch; s.max_ctx = cfg->max_ctx; s.eps = cfg->rms_eps; s.has_bias = cfg->qkv_bias ? 1 : 0;
  s.R_ffn = tile_rows(s.F);
  s.R_qkv = qkv_tile_rows(s.RQKV / 2);
}

extern "C" int easyspec_create(const easyspec_config* cfg, void* hip_stream, easyspec_ctx** out) {
  if (!out) return fail(nullptr, EASYSPEC_EINVAL, "out is NULL");
  *out = nullptr;
  int rc = check_config(cfg);
  if (rc != EASYSPEC_OK) return rc;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1)
    return fail(nullptr, EASYSPEC_EHIP, "no HIP device available (this library has no CPU path)");

  easyspec_ctx* ctx = new easyspec_ctx();
  ctx->cfg = *cfg;
  ctx->stream = (hipStream_t)hip_stream;
  ctx->weights_loaded = false;
  ctx->last_rows = 0;
  ctx->last_H = nullptr;
  ctx->has_b2 = false;
  ctx->prof_op = -1;
  ctx->timer = LaunchTimer{nullptr, nullptr, 0, 0, 0};
  ctx->parallel_mode = EASYSPEC_PARALLEL_ATTENTION;
  Shape& s = ctx->s;
  shape_of(cfg, s);
  ctx->precise.assign(s.B, 0);
  ctx->fuzzy.assign(s.B, 0);
  ctx->tree.assign(s.B, easyspec_ctx::Tree());
  for (int i = 0; i <= s.L; ++i) ctx->single.push_back(i);
  ctx->bounds = ctx->single;

  auto body = [&]() -> int {
    Buffers& b = ctx->b;
    memset(&b, 0, sizeof b);
    const size_t es_ = esize(s);
    const size_t act_ = es_ * (s.dtype == EASYSPEC_DTYPE_BF16 ? 2 : 1);  // bf16 activations: hi and lo arrays
    ALLOC(ctx, b.wqkv, (size_t)s.L * 2 * packed_bytes(s, s.RQKV / 2, s.d, s.R_qkv));
    ALLOC(ctx, b.wo, (size_t)s.L * packed_bytes(s, s.d, s.HQ));
    ALLOC(ctx, b.wg, (size_t)s.L * packed_bytes(s, s.F, s.d, s.R_ffn));
    ALLOC(ctx, b.wu, (size_t)s.L * packed_bytes(s, s.F, s.d, s.R_ffn));
    ALLOC(ctx, b.wd, (size_t)s.L * packed_bytes(s, s.d, s.F));
    ALLOC(ctx, b.wlm, packed_bytes(s, s.V, s.d));
    ALLOC(ctx, b.embed, (size_t)s.V * s.d * es_);
    if (s.has_bias) ALLOC(ctx, b.bqkv, (size_t)s.L * s.RQKV * sizeof(float));
    ALLOC(ctx, b.g_attn, (size_t)s.L * s.d * sizeof(float));
    ALLOC(ctx, b.g_mlp, (size_t)s.L * s.d * sizeof(float));
    ALLOC(ctx, b.g_final, (size_t)s.d * sizeof(float));
    ALLOC(ctx, b.rope, (size_t)s.max_ctx * (s.hd / 2) * sizeof(float2));
    const size_t kv_bytes = (size_t)s.L * s.B * s.Hkv * s.max_ctx * s.hd * es_;
    ALLOC(ctx, b.kc, kv_bytes);
    ALLOC(ctx, b.vc, kv_bytes);
    ALLOC_WORK(ctx, b.H, (size_t)kMaxCols * s.d * sizeof(float));
    ALLOC_WORK(ctx, b.ssp, (size_t)kMaxCols * (s.d / 16) * sizeof(float));
    ALLOC_WORK(ctx, b.XA, (size_t)EASYSPEC_MAX_SET * kMaxCols * s.d * act_);
    ALLOC_WORK(ctx, b.ssp_set, (size_t)EASYSPEC_MAX_SET * kMaxCols * (s.d / 16) * sizeof(float));
    ALLOC_WORK(ctx, b.XM, (size_t)EASYSPEC_MAX_SET * kMaxCols * s.d * act_);
    ALLOC_WORK(ctx, b.Q, (size_t)EASYSPEC_MAX_SET * kMaxCols * s.HQ * sizeof(float));
    ALLOC_WORK(ctx, b.AO, (size_t)EASYSPEC_MAX_SET * kMaxCols * s.HQ * act_);
    ALLOC_WORK(ctx, b.A, (size_t)EASYSPEC_MAX_SET * kMaxCols * s.d * sizeof(float));
    ALLOC_WORK(ctx, b.ACT, (size_t)EASYSPEC_MAX_SET * kMaxCols * s.F * act_);
    const size_t prow = (size_t)EASYSPEC_MAX_SET * kMaxCols * s.Hq;
    ALLOC_WORK(ctx, b.PO, prow * kMaxChunks * s.hd * sizeof(float));
    ALLOC_WORK(ctx, b.PM, prow * kMaxChunks * sizeof(float));
    ALLOC_WORK(ctx, b.PL, prow * kMaxChunks * sizeof(float));
    const size_t nblk = (size_t)(s.V + 15) / 16;
    ALLOC_WORK(ctx, b.amax_val, kMaxCols * nblk * sizeof(float));
    ALLOC_WORK(ctx, b.amax_idx, kMaxCols * nblk * sizeof(int32_t));
    // A calibration of more columns than one pass holds runs its passes two at a time (the weight kernels serve
    // both from one read of the weights): the second pass of a pair works in a workspace set of its own.
    Buffers& b2 = ctx->b2;
    b2 = b;
    ctx->has_b2 = (long)s.B * cfg->max_calib_tokens > kMaxCols;
    if (ctx->has_b2) {
      ALLOC_WORK(ctx, b2.H, (size_t)kMaxCols * s.d * sizeof(float));
      ALLOC_WORK(ctx, b2.ssp, (size_t)kMaxCols * (s.d / 16) * sizeof(float));
      ALLOC_WORK(ctx, b2.XA, (size_t)kMaxCols * s.d * act_);
      ALLOC_WORK(ctx, b2.XM, (size_t)kMaxCols * s.d * act_);
      ALLOC_WORK(ctx, b2.Q, (size_t)kMaxCols * s.HQ * sizeof(float));
      ALLOC_WORK(ctx, b2.AO, (size_t)kMaxCols * s.HQ * act_);
      ALLOC_WORK(ctx, b2.A, (size_t)kMaxCols * s.d * sizeof(float));
      ALLOC_WORK(ctx, b2.ACT, (size_t)kMaxCols * s.F * act_);
      const size_t prow2 = (size_t)kMaxCols * s.Hq;  // calibrations go layer by layer: one layer's worth of each
      ALLOC_WORK(ctx, b2.PO, prow2 * kMaxChunks * s.hd * sizeof(float));
      ALLOC_WORK(ctx, b2.PM, prow2 * kMaxChunks * sizeof(float));
      ALLOC_WORK(ctx, b2.PL, prow2 * kMaxChunks * sizeof(float));
      ALLOC_WORK(ctx, b2.amax_val, kMaxCols * nblk * sizeof(float));
      ALLOC_WORK(ctx, b2.amax_idx, kMaxCols * nblk * sizeof(int32_t));
      b2.ssp_set = nullptr;  // full-layer mode never runs two passes together
    }
    HIPCHK(ctx, hipMemsetAsync(b.kc, 0, kv_bytes, ctx->stream));
    HIPCHK(ctx, hipMemsetAsync(b.vc, 0, kv_bytes, ctx->stream));

    // rotary table in double precision: angle(pos, i) = pos * theta^(-2 i / hd)
    const int half = s.hd / 2;
    std::vector<float2> tab((size_t)s.max_ctx * half);
    std::vector<double> freq(half);
    for (int i = 0; i < half; ++i) freq[i] = pow((double)cfg->rope_theta, -2.0 * (double)i / (double)s.hd);
    for (int p = 0; p < s.max_ctx; ++p)
      for (int i = 0; i < half; ++i) {
        const double ang = (double)p * freq[i];
        tab[(size_t)p * half + i] = make_float2((float)cos(ang), (float)sin(ang));
      }
    HIPCHK(ctx, hipMemcpy(b.rope, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice));
    HIPCHK(ctx, hipStreamSynchronize(ctx->stream));
    return EASYSPEC_OK;
  };
  rc = body();
  if (rc != EASYSPEC_OK) {
    g_err = ctx->err;
    for (void* p : ctx->allocs) (void)hipFree(p);
    delete ctx;
    return rc;
  }
  *out = ctx;
  return EASYSPEC_OK;
}

extern "C" void easyspec_destroy(easyspec_ctx* ctx) {
  if (!ctx) return;
  (void)hipStreamSynchronize(ctx->stream);
  for (hipEvent_t e : ctx->prof_ev) (void)hipEventDestroy(e);
  for (void* p : ctx->allocs) (void)hipFree(p);
  delete ctx;
}

extern "C" const char* easyspec_last_error(const easyspec_ctx* ctx) { return ctx ? ctx->err.c_str() : g_err.c_str(); }

// ---------------------------------------------------------------------------------------------
// weights
// ---------------------------------------------------------------------------------------------

extern "C" int easyspec_load_weights(easyspec_ctx* ctx, const easyspec_weights* w) {
  if (!ctx) return fail(nullptr, EASYSPEC_EINVAL, "ctx is NULL");
  if (!w || !w->layers || !w->embed || !w->lm_head || !w->g_final) return fail(ctx, EASYSPEC_EINVAL, "weights: NULL pointer");
  const Shape& s = ctx->s;
  for (int l = 0; l < s.L; ++l) {
    const easyspec_layer_weights& lw = w->layers[l];
    if (!lw.wq || !lw.wk || !lw.wv || !lw.wo || !lw.wg || !lw.wu || !lw.wd || !lw.g_attn || !lw.g_mlp)
      return fail(ctx, EASYSPEC_EINVAL, "weights: NULL pointer in layer %d", l);
    if (s.has_bias && (!lw.bq || !lw.bk || !lw.bv)) return fail(ctx, EASYSPEC_EINVAL, "weights: missing bias in layer %d", l);
  }
  const size_t es_ = esize(s);
  const Buffers& b = ctx->b;
  // staging for one row-major matrix (largest: LM head, gate/up, or stacked QKV)
  size_t stage_elems = (size_t)s.V * s.d;
  if ((size_t)s.F * s.d > stage_elems) stage_elems = (size_t)s.F * s.d;
  if ((size_t)s.RQKV * s.d > stage_elems) stage_elems = (size_t)s.RQKV * s.d;
  void* stage = nullptr;
  HIPCHK(ctx, hipMalloc(&stage, stage_elems * es_));
  auto body = [&]() -> int {
    hipStream_t st = ctx->stream;
    auto put = [&](const void* src, size_t elems, size_t off_elems) -> hipError_t {
      return hipMemcpyAsync((char*)stage + off_elems * es_, src, elems * es_, hipMemcpyDefault, st);
    };
    auto pack = [&](void* dst_base, size_t layer, int rows, int K, int R = 16) -> hipError_t {
      launch_repack(s.dtype, stage, (char*)dst_base + layer * packed_bytes(s, rows, K, R), rows, K, R, 0, 0, st);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
      return hipStreamSynchronize(st);  // staging is reused
    };
    // stacked [Wq; Wk; Wv]: the first halves of all heads, then the second halves (the rotation pairs)
    auto pack_qkv = [&](size_t layer) -> hipError_t {
      const size_t half_bytes = packed_bytes(s, s.RQKV / 2, s.d, s.R_qkv);
      char* dst = (char*)b.wqkv + layer * 2 * half_bytes;
      launch_repack(s.dtype, stage, dst, s.RQKV / 2, s.d, s.R_qkv, s.hd / 2, 0, st);
      launch_repack(s.dtype, stage, dst + half_bytes, s.RQKV / 2, s.d, s.R_qkv, s.hd / 2, s.hd / 2, st);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
      return hipStreamSynchronize(st);
    };
    for (int l = 0; l < s.L; ++l) {
      const easyspec_layer_weights& lw = w->layers[l];
      HIPCHK(ctx, put(lw.wq, (size_t)s.HQ * s.d, 0));
      HIPCHK(ctx, put(lw.wk, (size_t)s.Hkv * s.hd * s.d, (size_t)s.HQ * s.d));
      HIPCHK(ctx, put(lw.wv, (size_t)s.Hkv * s.hd * s.d, (size_t)(s.HQ + s.Hkv * s.hd) * s.d));
      HIPCHK(ctx, pack_qkv(l));
      HIPCHK(ctx, put(lw.wo, (size_t)s.d * s.HQ, 0));
      HIPCHK(ctx, pack(b.wo, l, s.d, s.HQ));
      HIPCHK(ctx, put(lw.wg, (size_t)s.F * s.d, 0));
      HIPCHK(ctx, pack(b.wg, l, s.F, s.d, s.R_ffn));
      HIPCHK(ctx, put(lw.wu, (size_t)s.F * s.d, 0));
      HIPCHK(ctx, pack(b.wu, l, s.F, s.d, s.R_ffn));
      HIPCHK(ctx, put(lw.wd, (size_t)s.d * s.F, 0));
      HIPCHK(ctx, pack(b.wd, l, s.d, s.F));
      if (s.has_bias) {
        float* dst = b.bqkv + (size_t)l * s.RQKV;
        HIPCHK(ctx, hipMemcpyAsync(dst, lw.bq, (size_t)s.HQ * 4, hipMemcpyDefault, st));
        HIPCHK(ctx, hipMemcpyAsync(dst + s.HQ, lw.bk, (size_t)s.Hkv * s.hd * 4, hipMemcpyDefault, st));
        HIPCHK(ctx, hipMemcpyAsync(dst + s.HQ + s.Hkv * s.hd, lw.bv, (size_t)s.Hkv * s.hd * 4, hipMemcpyDefault, st));
      }
      HIPCHK(ctx, hipMemcpyAsync(b.g_attn + (size_t)l * s.d, lw.g_attn, (size_t)s.d * 4, hipMemcpyDefault, st));
      HIPCHK(ctx, hipMemcpyAsync(b.g_mlp + (size_t)l * s.d, lw.g_mlp, (size_t)s.d * 4, hipMemcpyDefault, st));
    }
    HIPCHK(ctx, put(w->lm_head, (size_t)s.V * s.d, 0));
    HIPCHK(ctx, pack(b.wlm, 0, s.V, s.d));
    HIPCHK(ctx, hipMemcpyAsync(b.embed, w->embed, (size_t)s.V * s.d * es_, hipMemcpyDefault, st));
    HIPCHK(ctx, hipMemcpyAsync(b.g_final, w->g_final, (size_t)s.d * 4, hipMemcpyDefault, st));
    HIPCHK(ctx, hipStreamSynchronize(st));
    return EASYSPEC_OK;
  };
  const int rc = body();
  (void)hipFree(stage);
  if (rc == EASYSPEC_OK) ctx->weights_loaded = true;
  return rc;
}

// ---------------------------------------------------------------------------------------------
// layer-parallel strategy
// ---------------------------------------------------------------------------------------------

extern "C" int easyspec_default_groups(int32_t L, int32_t N, int32_t policy, int32_t* bounds, int32_t* n_sets) {
  if (L < 1 || N < 1 || !bounds || !n_sets) return fail(nullptr, EASYSPEC_EINVAL, "default_groups: bad arguments");
  if (policy != EASYSPEC_POLICY_ALIGNED && policy != EASYSPEC_POLICY_PACKED) return fail(nullptr, EASYSPEC_EINVAL, "default_groups: unknown policy %d", policy);
  std::vector<int32_t> b;
  b.push_back(0);
  if (L >= 2) {
    // layers 1 .. L-2 are cut into N-sets; layer 0 and layer L-1 stay alone
    const int32_t stop = L - 1;
    int32_t lo = 1;
    b.push_back(lo);
    while (lo < stop) {
      int32_t hi = policy == EASYSPEC_POLICY_ALIGNED ? (lo / N + 1) * N : lo + N;
      if (hi > stop) hi = stop;
      b.push_back(hi);
      lo = hi;
    }
  }
  b.push_back(L);
  for (size_t i = 0; i < b.size(); ++i) bounds[i] = b[i];
  *n_sets = (int32_t)b.size() - 1;
  return EASYSPEC_OK;
}

extern "C" int easyspec_set_groups(easyspec_ctx* ctx, const int32_t* bounds, int32_t n_sets) {
  if (!ctx) return fail(nullptr, EASYSPEC_EINVAL, "ctx is NULL");
  if (!bounds || n_sets < 1 || n_sets > ctx->s.L) return fail(ctx, EASYSPEC_EINVAL, "set_groups: bad n_sets");
  if (bounds[0] != 0 || bounds[n_sets] != ctx->s.L) return fail(ctx, EASYSPEC_EINVAL, "set_groups: bounds must run from 0 to n_layers");
  for (int j = 0; j < n_sets; ++j) {
    const int k = bounds[j + 1] - bounds[j];
    if (k < 1) return fail(ctx, EASYSPEC_EINVAL, "set_groups: bounds must increase");
    if (k > EASYSPEC_MAX_SET) return fail(ctx, EASYSPEC_EINVAL, "set_groups: set of %d layers exceeds %d", k, EASYSPEC_MAX_SET);
  }
  ctx->bounds.assign(bounds, bounds + n_sets + 1);
  return EASYSPEC_OK;
}

// ---------------------------------------------------------------------------------------------
// one forward pass over the columns `c` (launch sequence of Alg. 1 / Alg. 2)
// ---------------------------------------------------------------------------------------------

// While profiling is on, the launches of one kernel class made inside the scope take event pairs.
struct ProfScope {
  ProfScope(easyspec_ctx* c, int op) {
    g_launch_timer = (c->prof_op == op || c->prof_op == EASYSPEC_OP_ALL) ? &c->timer : nullptr;
    c->timer.cur_op = op;
  }
  ~ProfScope() { g_launch_timer = nullptr; }
};

// c2: a second pass of as many columns run together with the first (sets of one layer only: a calibration); the
// weight kernels then serve both passes in one launch each, embedding, attention and argmax run per pass.
static int forward(easyspec_ctx* ctx, const Cols& c, const int32_t* tokens, const std::vector<int32_t>& bounds,
                   bool full_layer, float* logits_out, int32_t* tokens_out, const Cols* c2 = nullptr) {
  const Shape& s = ctx->s;
  const Buffers& b = ctx->b;
  const Buffers* b2 = c2 ? &ctx->b2 : nullptr;
  hipStream_t st = ctx->stream;
  const int n_sets = (int)bounds.size() - 1;
  if (c2 && (full_layer || !ctx->has_b2 || c2->n != c.n || n_sets != s.L))
    return fail(ctx, EASYSPEC_EINVAL, "internal: two passes together need equal column counts and sets of one layer");
  { ProfScope p(ctx, EASYSPEC_OP_ALL); launch_embed(s, b, c, tokens, 0, bounds[1] - bounds[0], st); }
  if (c2) { ProfScope p(ctx, EASYSPEC_OP_ALL); launch_embed(s, *b2, *c2, tokens, 0, 1, st); }
  for (int j = 0; j < n_sets; ++j) {
    const int lo = bounds[j], hi = bounds[j + 1], k = hi - lo;
    const AttnCut cut = attn_cut(s, c, k);
    // every attention layer of the set reads the hidden state that enters the set
    { ProfScope p(ctx, EASYSPEC_OP_QKV); launch_qkv(s, b, c, lo, k, st, b2, c2); }
    { ProfScope p(ctx, EASYSPEC_OP_ATTN); launch_attn(s, b, c, lo, k, cut, st); }
    if (c2) { ProfScope p(ctx, EASYSPEC_OP_ATTN); launch_attn(s, *b2, *c2, lo, k, attn_cut(s, *c2, k), st); }
    if (full_layer && k > 1) {
      // App. B ablation: the MLPs of the set also work from the set's input, each behind its own
      // layer's attention; one launch per operation for the whole set
      { ProfScope p(ctx, EASYSPEC_OP_OPROJ); launch_oproj_full(s, b, c, lo, k, st); }
      { ProfScope p(ctx, EASYSPEC_OP_GATEUP); launch_gateup(s, b, c, lo, k, b.ssp_set, st); }
      ProfScope p(ctx, EASYSPEC_OP_DOWN);
      if (hi < s.L) launch_down_full(s, b, c, lo, k, b.g_attn + (size_t)hi * s.d, bounds[j + 2] - hi, b.XA, st);
      else launch_down_full(s, b, c, lo, k, b.g_final, 1, b.XA, st);
      continue;
    }
    { ProfScope p(ctx, EASYSPEC_OP_OPROJ); launch_oproj(s, b, c, lo, k, st, b2, c2); }
    // the MLPs run in layer order on the running residual
    for (int i = lo; i < hi; ++i) {
      { ProfScope p(ctx, EASYSPEC_OP_GATEUP); launch_gateup(s, b, c, i, 1, b.ssp, st, b2, c2, c2 ? b2->ssp : nullptr); }
      ProfScope p(ctx, EASYSPEC_OP_DOWN);
      if (i + 1 < hi) {
        launch_down(s, b, c, i, i + 1 - lo, b.g_mlp + (size_t)(i + 1) * s.d, 1, b.XM, st, b2, c2, c2 ? b2->XM : nullptr);
      } else if (hi < s.L) {
        launch_down(s, b, c, i, -1, b.g_attn + (size_t)hi * s.d, bounds[j + 2] - hi, b.XA, st, b2, c2, c2 ? b2->XA : nullptr);
      } else {
        launch_down(s, b, c, i, -1, b.g_final, 1, b.XA, st, b2, c2, c2 ? b2->XA : nullptr);
      }
    }
  }
  { ProfScope p(ctx, EASYSPEC_OP_HEAD); launch_head(s, b, c, logits_out, tokens_out, st, b2, c2); }
  HIPCHK(ctx, hipGetLastError());
  ctx->last_rows = c2 ? c2->n : c.n;
  ctx->last_H = c2 ? b2->H : b.H;
  return EASYSPEC_OK;
}

extern "C" int easyspec_set_parallel_mode(easyspec_ctx* ctx, int32_t mode) {
  if (!ctx) return fail(nullptr, EASYSPEC_EINVAL, "ctx is NULL");
  if (mode != EASYSPEC_PARALLEL_ATTENTION && mode != EASYSPEC_PARALLEL_FULL_LAYER)
    return fail(ctx, EASYSPEC_EINVAL, "set_parallel_mode: unknown mode %d", mode);
  ctx->parallel_mode = mode;
  return EASYSPEC_OK;
}

extern "C" int easyspec_draft_step(easyspec_ctx* ctx, const int32_t* tokens_in, int32_t* tokens_out, float* logits_out) {
  if (!ctx) return fail(nullptr, EASYSPEC_EINVAL, "ctx is NULL");
  if (!ctx->weights_loaded) return fail(ctx, EASYSPEC_ESTATE, "draft_step: no weights loaded");
  if (!tokens_in || !tokens_out) return fail(ctx, EASYSPEC_EINVAL, "draft_step: NULL token array");
  const Shape& s = ctx->s;
  Cols c;
  memset(&c, 0, sizeof c);
  for (int b = 0; b < s.B; ++b) {
    if (ctx->precise[b] == 0) continue;
    const int pos = ctx->precise[b] + ctx->fuzzy[b];
    if (pos + 1 > s.max_ctx) return fail(ctx, EASYSPEC_ECAPACITY, "draft_step: sequence %d is full (%d slots)", b, s.max_ctx);
    if (ctx->tree[b].n > 0) return fail(ctx, EASYSPEC_ESTATE, "draft_step: sequence %d holds a token tree (continue it with easyspec_draft_tree_step)", b);
    c.seq[c.n] = b; c.pos[c.n] = pos; c.tok_idx[c.n] = b; c.logit_row[c.n] = b; c.out_idx[c.n] = b;
    c.rope_pos[c.n] = pos; c.vis_base[c.n] = pos + 1;  // causal: every earlier slot is visible
    ++c.n;
  }
  if (c.n == 0) return fail(ctx, EASYSPEC_ESTATE, "draft_step: no live sequence (calibrate a prompt first)");
  const int rc = forward(ctx, c, tokens_in, ctx->bounds, ctx->parallel_mode == EASYSPEC_PARALLEL_FULL_LAYER, logits_out, tokens_out);
  if (rc != EASYSPEC_OK) return rc;
  for (int i = 0; i < c.n; ++i) ctx->fuzzy[c.seq[i]] += 1;
  return EASYSPEC_OK;
}

extern "C" int easyspec_draft_tree_step(easyspec_ctx* ctx, const int32_t* tokens_in, const int32_t* n_nodes, const int32_t* parents,
                                        int32_t* tokens_out, float* logits_out) {
  if (!ctx) return fail(nullptr, EASYSPEC_EINVAL, "ctx is NULL");
  if (!ctx->weights_loaded) return fail(ctx, EASYSPEC_ESTATE, "draft_tree_step: no weights loaded");
  if (!tokens_in || !n_nodes || !parents || !tokens_out) return fail(ctx, EASYSPEC_EINVAL, "draft_tree_step: NULL argument");
  const Shape& s = ctx->s;
  const int W = EASYSPEC_MAX_TREE_WIDTH;
  Cols c;
  memset(&c, 0, sizeof c);
  for (int b = 0; b < s.B; ++b) {
    const int n = n_nodes[b];
    if (n == 0) continue;
    const easyspec_ctx::Tree& t = ctx->tree[b];
    if (n < 0 || n > W) return fail(ctx, EASYSPEC_EINVAL, "draft_tree_step: n_nodes[%d] = %d outside 0..%d", b, n, W);
    if (ctx->precise[b] == 0) return fail(ctx, EASYSPEC_ESTATE, "draft_tree_step: sequence %d has no context (calibrate a prompt first)", b);
    if (ctx->fuzzy[b] != t.n) return fail(ctx, EASYSPEC_ESTATE, "draft_tree_step: sequence %d holds chain-drafted slots; calibrate first", b);
    if (t.n + n > EASYSPEC_MAX_TREE_NODES) return fail(ctx, EASYSPEC_ECAPACITY, "draft_tree_step: sequence %d would hold %d > %d tree nodes", b, t.n + n, EASYSPEC_MAX_TREE_NODES);
    if (ctx->precise[b] + t.n + n > s.max_ctx) return fail(ctx, EASYSPEC_ECAPACITY, "draft_tree_step: sequence %d is full (%d slots)", b, s.max_ctx);
    if (c.n + n > kMaxCols) return fail(ctx, EASYSPEC_ECAPACITY, "draft_tree_step: more than %d nodes in one call", kMaxCols);
    for (int j = 0; j < n; ++j) {
      const int par = parents[b * W + j];
      if (par < -1 || par >= t.n) return fail(ctx, EASYSPEC_EINVAL, "draft_tree_step: parent %d of node %d of sequence %d is not a node of an earlier level", par, j, b);
      const int node = t.n + j;
      const int depth = par < 0 ? 0 : t.depth[par] + 1;
      c.seq[c.n] = b;
      c.pos[c.n] = ctx->precise[b] + node;
      c.rope_pos[c.n] = ctx->precise[b] + depth;
      c.vis_base[c.n] = ctx->precise[b];
      c.vis_mask[c.n] = (par < 0 ? 0ull : t.line[par]) | (1ull << node);
      c.tok_idx[c.n] = b * W + j; c.logit_row[c.n] = b * W + j; c.out_idx[c.n] = b * W + j;
      ++c.n;
    }
  }
  if (c.n == 0) return fail(ctx, EASYSPEC_EINVAL, "draft_tree_step: no nodes");
  const int rc = forward(ctx, c, tokens_in, ctx->bounds, ctx->parallel_mode == EASYSPEC_PARALLEL_FULL_LAYER, logits_out, tokens_out);
  if (rc != EASYSPEC_OK) return rc;
  for (int i = 0; i < c.n; ++i) {
    easyspec_ctx::Tree& t = ctx->tree[c.seq[i]];
    const int node = c.pos[i] - ctx->precise[c.seq[i]];
    t.depth[node] = c.rope_pos[i] - ctx->precise[c.seq[i]];
    t.line[node] = c.vis_mask[i];
  }
  for (int b = 0; b < s.B; ++b) {
    ctx->tree[b].n += n_nodes[b];
    ctx->fuzzy[b] += n_nodes[b];
  }
  return EASYSPEC_OK;
}

extern "C" int easyspec_calibrate(easyspec_ctx* ctx, const int32_t* tokens, const int32_t* n_tokens, int32_t* next_token_out,
                                  float* logits_out, int32_t logits_rows) {
  if (!ctx) return fail(nullptr, EASYSPEC_EINVAL, "ctx is NULL");
  if (!ctx->weights_loaded) return fail(ctx, EASYSPEC_ESTATE, "calibrate: no weights loaded");
  if (!tokens || !n_tokens || !next_token_out) return fail(ctx, EASYSPEC_EINVAL, "calibrate: NULL argument");
  if (logits_rows != 0 && logits_rows != 1) return fail(ctx, EASYSPEC_EINVAL, "calibrate: logits_rows must be 0 or 1");
  const Shape& s = ctx->s;
  const int mc = ctx->cfg.max_calib_tokens;
  int total = 0;
  for (int b = 0; b < s.B; ++b) {
    const int n = n_tokens[b];
    if (n < 0 || n > mc) return fail(ctx, EASYSPEC_ECAPACITY, "calibrate: n_tokens[%d] = %d outside 0..%d", b, n, mc);
    if (n > 0 && ctx->precise[b] + n > s.max_ctx)
      return fail(ctx, EASYSPEC_ECAPACITY, "calibrate: sequence %d would hold %d > %d slots", b, ctx->precise[b] + n, s.max_ctx);
    total += n;
  }
  if (total == 0) return fail(ctx, EASYSPEC_EINVAL, "calibrate: no tokens");
  // passes of at most 16 columns; a sequence's tokens stay together.  Two consecutive passes of equal column
  // counts run together, so that the weights are read once for both.
  int b = 0;
  Cols held;  // a pass waiting for a partner
  memset(&held, 0, sizeof held);
  bool holding = false;
  const char* pair_env = getenv("EASYSPEC_PAIR_PASSES");  // tests: 0 = one pass at a time; read at every call
  const bool pair_passes = !pair_env || atoi(pair_env) != 0;
  auto run = [&](const Cols& c, const Cols* partner) { return forward(ctx, c, tokens, ctx->single, false, logits_out, next_token_out, partner); };
  while (b < s.B) {
    Cols c;
    memset(&c, 0, sizeof c);
    while (b < s.B && c.n + n_tokens[b] <= kMaxCols) {
      const int n = n_tokens[b];
      for (int r = 0; r < n; ++r) {
        const bool last = r == n - 1;
        c.seq[c.n] = b;
        c.pos[c.n] = ctx->precise[b] + r;  // fuzzy slots are dropped: positions restart at the precise length
        c.rope_pos[c.n] = c.pos[c.n];
        c.vis_base[c.n] = c.pos[c.n] + 1;  // causal among the tokens of the pass
        c.tok_idx[c.n] = b * mc + r;
        c.logit_row[c.n] = logits_rows ? b * mc + r : (last ? b : -1);
        c.out_idx[c.n] = last ? b : -1;
        ++c.n;
      }
      ++b;
    }
    if (c.n == 0) continue;
    int rc = EASYSPEC_OK;
    if (holding && held.n == c.n) {
      rc = run(held, &c);
      holding = false;
    } else {
      if (holding) rc = run(held, nullptr);
      const bool more = b < s.B;  // sequences left: a partner may follow
      if (rc == EASYSPEC_OK && more && pair_passes && ctx->has_b2 && twin_passes_fit(s, c.n)) {
        held = c;
        holding = true;
      } else if (rc == EASYSPEC_OK) {
        holding = false;
        rc = run(c, nullptr);
      }
    }
    if (rc != EASYSPEC_OK) return rc;
  }
  if (holding) {
    const int rc = run(held, nullptr);
    if (rc != EASYSPEC_OK) return rc;
  }
  for (int q = 0; q < s.B; ++q)
    if (n_tokens[q] > 0) {
      ctx->fuzzy[q] = 0;
      ctx->tree[q].n = 0;
      ctx->precise[q] += n_tokens[q];
    }
  return EASYSPEC_OK;
}

// ---------------------------------------------------------------------------------------------
// acceptance, lengths, cache access
// ---------------------------------------------------------------------------------------------

static int check_greedy_args(const int32_t* draft, const int32_t* target, int32_t batch, int32_t gamma, int32_t* accept_len,
                             int32_t* bonus) {
  if (!target || !accept_len || !bonus || (gamma > 0 && !draft)) return fail(nullptr, EASYSPEC_EINVAL, "greedy_accept: NULL argument");
  if (batch < 1 || gamma < 0) return fail(nullptr, EASYSPEC_EINVAL, "greedy_accept: batch must be >= 1 and gamma >= 0");
  return EASYSPEC_OK;
}

extern "C" int easyspec_greedy_accept(const int32_t* draft, const int32_t* target, int32_t batch, int32_t gamma,
                                      int32_t* accept_len, int32_t* bonus, void* hip_stream) {
  const int rc = check_greedy_args(draft, target, batch, gamma, accept_len, bonus);
  if (rc != EASYSPEC_OK) return rc;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return fail(nullptr, EASYSPEC_EHIP, "no HIP device available (this library has no CPU path)");
  // a host array here would be written by the kernel through an address the device does not have
  hipPointerAttribute_t attr;
  if (hipPointerGetAttributes(&attr, accept_len) != hipSuccess || (attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeManaged)) {
    (void)hipGetLastError();
    return fail(nullptr, EASYSPEC_EINVAL, "greedy_accept: accept_len is not device memory (host arrays: easyspec_greedy_accept_host)");
  }
  launch_accept(draft, target, batch, gamma, accept_len, bonus, (hipStream_t)hip_stream);
  HIPCHK(nullptr, hipGetLastError());
  return EASYSPEC_OK;
}

extern "C" int easyspec_greedy_accept_host(const int32_t* draft, const int32_t* target, int32_t batch, int32_t gamma,
                                           int32_t* accept_len, int32_t* bonus) {
  const int rc = check_greedy_args(draft, target, batch, gamma, accept_len, bonus);
  if (rc != EASYSPEC_OK) return rc;
  for (int b = 0; b < batch; ++b) {
    const int32_t* d = draft + (size_t)b * gamma;
    const int32_t* t = target + (size_t)b * (gamma + 1);
    int m = 0;
    while (m < gamma && d[m] == t[m]) ++m;
    accept_len[b] = m;
    bonus[b] = t[m];
  }
  return EASYSPEC_OK;
}

extern "C" int64_t easyspec_accept_workspace_bytes(int32_t batch, int32_t gamma, int32_t vocab) {
  if (batch < 1 || gamma < 0 || vocab < 1) return -1;
  return (int64_t)sample_accept_workspace_bytes(batch, gamma, vocab);
}

static int check_accept_args(const int32_t* draft, const float* draft_logits, const float* target_logits, const float* r,
                             const float* u, int32_t batch, int32_t gamma, int32_t vocab, float temperature, int32_t* accept_len,
                             int32_t* bonus) {
  if (!target_logits || !u || !accept_len || !bonus) return fail(nullptr, EASYSPEC_EINVAL, "accept: NULL argument");
  if (gamma > 0 && (!draft || !draft_logits || !r)) return fail(nullptr, EASYSPEC_EINVAL, "accept: NULL draft argument with gamma > 0");
  if (batch < 1 || batch > 65535 || gamma < 0 || gamma > 64 || vocab < 1)
    return fail(nullptr, EASYSPEC_EINVAL, "accept: need 1 <= batch <= 65535, 0 <= gamma <= 64, vocab >= 1");
  if (!(temperature > 0.f) || !(temperature < INFINITY)) return fail(nullptr, EASYSPEC_EINVAL, "accept: temperature must be positive and finite (use easyspec_greedy_accept at 0)");
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return fail(nullptr, EASYSPEC_EHIP, "no HIP device available (this library has no CPU path)");
  return EASYSPEC_OK;
}

extern "C" int easyspec_accept(const int32_t* draft, const float* draft_logits, const float* target_logits, const float* r,
                               const float* u, int32_t batch, int32_t gamma, int32_t vocab, float temperature,
                               int32_t* accept_len, int32_t* bonus, void* workspace, void* hip_stream) {
  if (!workspace) return fail(nullptr, EASYSPEC_EINVAL, "accept: NULL argument");
  const int rc = check_accept_args(draft, draft_logits, target_logits, r, u, batch, gamma, vocab, temperature, accept_len, bonus);
  if (rc != EASYSPEC_OK) return rc;
  launch_sample_accept(draft, draft_logits, target_logits, r, u, batch, gamma, vocab, (double)temperature, (double*)workspace,
                       accept_len, bonus, (hipStream_t)hip_stream);
  HIPCHK(nullptr, hipGetLastError());
  return EASYSPEC_OK;
}

extern "C" int64_t easyspec_accept_static_max_bytes(void) { return (int64_t)sample_accept_static_capacity_bytes(); }

extern "C" int easyspec_accept_static(const int32_t* draft, const float* draft_logits, const float* target_logits, const float* r,
                                      const float* u, int32_t batch, int32_t gamma, int32_t vocab, float temperature,
                                      int32_t* accept_len, int32_t* bonus, void* hip_stream) {
  const int rc = check_accept_args(draft, draft_logits, target_logits, r, u, batch, gamma, vocab, temperature, accept_len, bonus);
  if (rc != EASYSPEC_OK) return rc;
  const size_t need = sample_accept_workspace_bytes(batch, gamma, vocab), have = sample_accept_static_capacity_bytes();
  if (need > have)
    return fail(nullptr, EASYSPEC_ECAPACITY, "accept_static: batch %d, gamma %d, vocab %d need %zu workspace bytes, the built-in workspace holds %zu (use easyspec_accept with a workspace of your own)",
                batch, gamma, vocab, need, have);
  double* ws = nullptr;
  HIPCHK(nullptr, sample_accept_static_workspace(&ws));
  // every workspace entry a call reads was written earlier in the same call, so nothing needs clearing
  launch_sample_accept(draft, draft_logits, target_logits, r, u, batch, gamma, vocab, (double)temperature, ws, accept_len, bonus,
                       (hipStream_t)hip_stream);
  HIPCHK(nullptr, hipGetLastError());
  return EASYSPEC_OK;
}

extern "C" int easyspec_get_lens(const easyspec_ctx* ctx, int32_t* precise, int32_t* fuzzy) {
  if (!ctx) return fail(nullptr, EASYSPEC_EINVAL, "ctx is NULL");
  for (int b = 0; b < ctx->s.B; ++b) {
    if (precise) precise[b] = ctx->precise[b];
    if (fuzzy) fuzzy[b] = ctx->fuzzy[b];
  }
  return EASYSPEC_OK;
}

extern "C" int easyspec_truncate(easyspec_ctx* ctx, int32_t b, int32_t new_len) {
  if (!ctx) return fail(nullptr, EASYSPEC_EINVAL, "ctx is NULL");
  if (b < 0 || b >= ctx->s.B) return fail(ctx, EASYSPEC_EINVAL, "truncate: sequence %d out of range", b);
  if (new_len < 0 || new_len > ctx->precise[b]) return fail(ctx, EASYSPEC_EINVAL, "truncate: length %d outside 0..%d", new_len, ctx->precise[b]);
  ctx->precise[b] = new_len;
  ctx->fuzzy[b] = 0;
  ctx->tree[b].n = 0;
  return EASYSPEC_OK;
}

static int kv_xfer(easyspec_ctx* ctx, int32_t b, void* k, void* v, int32_t n, int to_cache) {
  const Shape& s = ctx->s;
  const size_t bytes = (size_t)s.L * s.Hkv * n * s.hd * esize(s);
  if (bytes == 0) return EASYSPEC_OK;
  void *dk = nullptr, *dv = nullptr;
  HIPCHK(ctx, hipMalloc(&dk, bytes));
  if (hipMalloc(&dv, bytes) != hipSuccess) {
    (void)hipFree(dk);
    return fail(ctx, EASYSPEC_EHIP, "kv transfer: out of device memory");
  }
  auto body = [&]() -> int {
    hipStream_t st = ctx->stream;
    if (to_cache) {
      HIPCHK(ctx, hipMemcpyAsync(dk, k, bytes, hipMemcpyDefault, st));
      HIPCHK(ctx, hipMemcpyAsync(dv, v, bytes, hipMemcpyDefault, st));
    }
    launch_kv_copy(s, ctx->b, b, dk, dv, n, to_cache, st);
    HIPCHK(ctx, hipGetLastError());
    if (!to_cache) {
      HIPCHK(ctx, hipMemcpyAsync(k, dk, bytes, hipMemcpyDefault, st));
      HIPCHK(ctx, hipMemcpyAsync(v, dv, bytes, hipMemcpyDefault, st));
    }
    HIPCHK(ctx, hipStreamSynchronize(st));
    return EASYSPEC_OK;
  };
  const int rc = body();
  (void)hipFree(dk);
  (void)hipFree(dv);
  return rc;
}

extern "C" int easyspec_kv_import(easyspec_ctx* ctx, int32_t b, const void* k, const void* v, int32_t n_slots) {
  if (!ctx) return fail(nullptr, EASYSPEC_EINVAL, "ctx is NULL");
  if (b < 0 || b >= ctx->s.B) return fail(ctx, EASYSPEC_EINVAL, "kv_import: sequence %d out of range", b);
  if (n_slots < 0 || n_slots > ctx->s.max_ctx) return fail(ctx, EASYSPEC_ECAPACITY, "kv_import: %d slots exceed max_ctx %d", n_slots, ctx->s.max_ctx);
  if (n_slots > 0 && (!k || !v)) return fail(ctx, EASYSPEC_EINVAL, "kv_import: NULL argument");
  const int rc = kv_xfer(ctx, b, const_cast<void*>(k), const_cast<void*>(v), n_slots, 1);
  if (rc != EASYSPEC_OK) return rc;
  ctx->precise[b] = n_slots;
  ctx->fuzzy[b] = 0;
  ctx->tree[b].n = 0;
  return EASYSPEC_OK;
}

extern "C" int easyspec_kv_export(easyspec_ctx* ctx, int32_t b, void* k, void* v, int32_t n_slots) {
  if (!ctx) return fail(nullptr, EASYSPEC_EINVAL, "ctx is NULL");
  if (b < 0 || b >= ctx->s.B) return fail(ctx, EASYSPEC_EINVAL, "kv_export: sequence %d out of range", b);
  if (n_slots < 0 || n_slots > ctx->s.max_ctx) return fail(ctx, EASYSPEC_ECAPACITY, "kv_export: %d slots exceed max_ctx %d", n_slots, ctx->s.max_ctx);
  if (n_slots > 0 && (!k || !v)) return fail(ctx, EASYSPEC_EINVAL, "kv_export: NULL argument");
  return kv_xfer(ctx, b, k, v, n_slots, 0);
}

extern "C" int easyspec_get_hidden(easyspec_ctx* ctx, float* out, int32_t max_rows, int32_t* n_rows) {
  if (!ctx) return fail(nullptr, EASYSPEC_EINVAL, "ctx is NULL");
  if (!out || !n_rows) return fail(ctx, EASYSPEC_EINVAL, "get_hidden: NULL argument");
  if (ctx->last_rows == 0) return fail(ctx, EASYSPEC_ESTATE, "get_hidden: no forward has run");
  if (max_rows < ctx->last_rows) return fail(ctx, EASYSPEC_ECAPACITY, "get_hidden: %d rows needed", ctx->last_rows);
  HIPCHK(ctx, hipMemcpyAsync(out, ctx->last_H, (size_t)ctx->last_rows * ctx->s.d * sizeof(float), hipMemcpyDeviceToDevice, ctx->stream));
  *n_rows = ctx->last_rows;
  return EASYSPEC_OK;
}

extern "C" int easyspec_poison_workspaces(easyspec_ctx* ctx) {
  if (!ctx) return fail(nullptr, EASYSPEC_EINVAL, "ctx is NULL");
  // all bits set: a NaN in float32 and in bf16, -1 as an index
  for (const auto& w : ctx->work) HIPCHK(ctx, hipMemsetAsync(w.first, 0xFF, w.second, ctx->stream));
  return EASYSPEC_OK;
}

extern "C" int easyspec_profile_begin(easyspec_ctx* ctx, int32_t op, int32_t max_launches) {
  if (!ctx) return fail(nullptr, EASYSPEC_EINVAL, "ctx is NULL");
  if (op < EASYSPEC_OP_QKV || op > EASYSPEC_OP_ALL) return fail(ctx, EASYSPEC_EINVAL, "profile_begin: unknown op %d", op);
  if (max_launches < 1 || max_launches > (1 << 20)) return fail(ctx, EASYSPEC_EINVAL, "profile_begin: bad max_launches");
  if (ctx->prof_op >= 0) return fail(ctx, EASYSPEC_ESTATE, "profile_begin: already profiling");
  while (ctx->prof_ev.size() < (size_t)max_launches * 2) {
    hipEvent_t e;
    HIPCHK(ctx, hipEventCreate(&e));
    ctx->prof_ev.push_back(e);
  }
  if (ctx->prof_op_of.size() < (size_t)max_launches) ctx->prof_op_of.resize((size_t)max_launches);
  ctx->timer = LaunchTimer{ctx->prof_ev.data(), ctx->prof_op_of.data(), (size_t)max_launches * 2, 0, 0};
  ctx->prof_op = op;
  return EASYSPEC_OK;
}

extern "C" int easyspec_profile_end(easyspec_ctx* ctx, int32_t* n_launches, float* total_ms, float* launch_ms, int32_t* launch_op) {
  if (!ctx) return fail(nullptr, EASYSPEC_EINVAL, "ctx is NULL");
  if (!n_launches || !total_ms) return fail(ctx, EASYSPEC_EINVAL, "profile_end: NULL argument");
  if (ctx->prof_op < 0) return fail(ctx, EASYSPEC_ESTATE, "profile_end: not profiling");
  ctx->prof_op = -1;
  HIPCHK(ctx, hipStreamSynchronize(ctx->stream));
  float sum = 0.f;
  for (size_t i = 0; i + 1 < ctx->timer.used; i += 2) {
    float ms = 0.f;
    HIPCHK(ctx, hipEventElapsedTime(&ms, ctx->timer.ev[i], ctx->timer.ev[i + 1]));
    if (launch_ms) launch_ms[i / 2] = ms;
    if (launch_op) launch_op[i / 2] = ctx->timer.op[i / 2];
    sum += ms;
  }
  *n_launches = (int32_t)(ctx->timer.used / 2);
  *total_ms = sum;
  return EASYSPEC_OK;
}

extern "C" int easyspec_stream_read(const void* buf, int64_t bytes, float* sink, void* hip_stream) {
  if (!buf || !sink) return fail(nullptr, EASYSPEC_EINVAL, "stream_read: NULL argument");
  if (bytes < 16 || bytes % 16 != 0) return fail(nullptr, EASYSPEC_EINVAL, "stream_read: bytes must be a positive multiple of 16");
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return fail(nullptr, EASYSPEC_EHIP, "no HIP device available (this library has no CPU path)");
  launch_stream_read(buf, (size_t)bytes, sink, (hipStream_t)hip_stream);
  HIPCHK(nullptr, hipGetLastError());
  return EASYSPEC_OK;
}

extern "C" int32_t easyspec_stream_read_sink_floats(void) { return stream_read_sink_floats(); }

static_assert(EASYSPEC_MAX_CHUNKS == kMaxChunks, "header and kernels disagree on the chunk limit");

extern "C" int easyspec_attention_cut(const easyspec_config* cfg, const int32_t* ctx_lens, int32_t n_cols, int32_t n_layers_in_set,
                                      int32_t* n_chunks, int32_t* ranges) {
  int rc = check_config(cfg);
  if (rc != EASYSPEC_OK) return rc;
  if (!ctx_lens || !n_chunks) return fail(nullptr, EASYSPEC_EINVAL, "attention_cut: NULL argument");
  if (n_cols < 1 || n_cols > kMaxCols) return fail(nullptr, EASYSPEC_EINVAL, "attention_cut: n_cols must be 1..%d", kMaxCols);
  if (n_layers_in_set < 1 || n_layers_in_set > EASYSPEC_MAX_SET)
    return fail(nullptr, EASYSPEC_EINVAL, "attention_cut: n_layers_in_set must be 1..%d", EASYSPEC_MAX_SET);
  Shape s;
  memset(&s, 0, sizeof s);
  s.dtype = cfg->dtype; s.Hq = cfg->n_q_heads; s.Hkv = cfg->n_kv_heads; s.hd = cfg->head_dim; s.max_ctx = cfg->max_ctx;
  Cols c;
  memset(&c, 0, sizeof c);
  c.n = n_cols;
  for (int i = 0; i < n_cols; ++i) {
    if (ctx_lens[i] < 1 || ctx_lens[i] > cfg->max_ctx)
      return fail(nullptr, EASYSPEC_EINVAL, "attention_cut: ctx_lens[%d] = %d outside 1..%d", i, ctx_lens[i], cfg->max_ctx);
    c.pos[i] = ctx_lens[i] - 1;
  }
  const AttnCut cut = attn_cut_vector(s, c, n_layers_in_set);
  const int nwv = attn_waves(cut);
  if (ranges) memset(ranges, 0, sizeof(int32_t) * (size_t)n_cols * EASYSPEC_MAX_CHUNKS * 8 * 2);
  for (int i = 0; i < n_cols; ++i) {
    int nch = 0, w0 = 0, w1 = 0;
    attn_ranges(s, cut, ctx_lens[i], 0, 0, &nch, &w0, &w1);
    n_chunks[i] = nch;
    if (!ranges) continue;
    for (int ch = 0; ch < nch && ch < EASYSPEC_MAX_CHUNKS; ++ch)
      for (int w = 0; w < nwv; ++w) {
        attn_ranges(s, cut, ctx_lens[i], ch, w, &nch, &w0, &w1);
        int32_t* r = ranges + (((size_t)i * EASYSPEC_MAX_CHUNKS + ch) * 8 + w) * 2;
        r[0] = w0;
        r[1] = w1;
      }
  }
  return nwv;
}

extern "C" int easyspec_attention_stage_walk(int32_t n_loads, int64_t* report) {
  if (!report) return fail(nullptr, EASYSPEC_EINVAL, "attention_stage_walk: NULL report");
  if (n_loads != 2 && n_loads != 8) return fail(nullptr, EASYSPEC_EINVAL, "attention_stage_walk: n_loads must be 2 or 8");
  constexpr int kPlaces = 32 * kStageRowPieces;  // 32 rows of 16 pieces = the 8 KB a wave owns
  int held_slot[kPlaces], held_piece[kPlaces], stores_at[kPlaces];
  for (int i = 0; i < kPlaces; ++i) held_slot[i] = held_piece[i] = -1, stores_at[i] = 0;
  int64_t* r = report;
  for (int i = 0; i < EASYSPEC_STAGE_FIELDS; ++i) r[i] = 0;
  r[3] = kPlaces;
  auto quarter_conflicts = [&](const int (&place)[64]) {
    int64_t n = 0;
    for (int q = 0; q < 4; ++q)
      for (int a = 0; a < 16; ++a)
        for (int b = a + 1; b < 16; ++b) n += (place[16 * q + a] & 15) == (place[16 * q + b] & 15);
    return n;
  };
  for (int j = 0; j < n_loads; ++j) {
    int place[64];
    for (int lane = 0; lane < 64; ++lane) {
      const int at = stage_store_piece(lane, j);
      place[lane] = at;
      ++r[0];
      if (at < 0 || at >= kPlaces) return fail(nullptr, EASYSPEC_EINVAL, "attention_stage_walk: store outside the stage");
      if (stores_at[at]++ == 0) ++r[1];
      held_slot[at] = 4 * j + (lane >> 4);
      held_piece[at] = lane & 15;
      r[2] = std::max<int64_t>(r[2], at + 1);
    }
    r[8] += quarter_conflicts(place);
  }
  const int n_tiles = (n_loads + 3) / 4;
  for (int t = 0; t < n_tiles; ++t)
    for (int kt = 0; kt < 4; ++kt) {
      int place[64];
      for (int lane = 0; lane < 64; ++lane) {
        const int at = stage_fetch_piece(lane, t, kt);
        place[lane] = at;
        if (at < 0 || at >= kPlaces) return fail(nullptr, EASYSPEC_EINVAL, "attention_stage_walk: fetch outside the stage");
        const int want_slot = t * 16 + stage_tile_slot(lane), want_piece = 4 * kt + (lane >> 4);
        if (want_slot >= 4 * n_loads) {
          ++r[6];
          continue;
        }
        ++r[4];
        r[5] += held_slot[at] != want_slot || held_piece[at] != want_piece;
      }
      r[8] += quarter_conflicts(place);
    }
  for (int j = 0; j < n_loads; ++j)
    for (int lane = 0; lane < 64; ++lane) {
      const int t = j / 4, i = j % 4;
      // element i of the lane's MFMA result is A row 4 (lane / 16) + i, fed by the lanes whose lane % 16 is that row
      const int a_row = 4 * (lane >> 4) + i;
      const int slot_of_row = t * 16 + stage_tile_slot(a_row);
      r[7] += slot_of_row != 4 * j + (lane >> 4) || score_slot_in_batch(lane, t, i) != 4 * j + (lane >> 4);
    }
  return EASYSPEC_OK;
}

extern "C" int easyspec_weight_walk(const easyspec_config* cfg, int32_t op, int32_t n_cols, int32_t n_layers_in_set, int32_t full_layer,
                                    int64_t* report) {
  int rc = check_config(cfg);
  if (rc != EASYSPEC_OK) return rc;
  if (!report) return fail(nullptr, EASYSPEC_EINVAL, "weight_walk: NULL argument");
  if (op != EASYSPEC_OP_QKV && op != EASYSPEC_OP_OPROJ && op != EASYSPEC_OP_GATEUP && op != EASYSPEC_OP_DOWN && op != EASYSPEC_OP_HEAD)
    return fail(nullptr, EASYSPEC_EINVAL, "weight_walk: op %d streams no packed matrix", op);
  if (n_cols < 1 || n_cols > kMaxCols) return fail(nullptr, EASYSPEC_EINVAL, "weight_walk: n_cols must be 1..%d", kMaxCols);
  if (n_layers_in_set < 1 || n_layers_in_set > EASYSPEC_MAX_SET || n_layers_in_set > cfg->n_layers)
    return fail(nullptr, EASYSPEC_EINVAL, "weight_walk: n_layers_in_set must be 1..%d and at most n_layers", EASYSPEC_MAX_SET);
  Shape s;
  shape_of(cfg, s);
  const StreamPlan p = stream_plan(s, op, n_cols, n_layers_in_set, full_layer != 0);
  StreamWalk w;
  if (stream_walk(s, p, n_cols, &w) != 0) return fail(nullptr, EASYSPEC_EINVAL, "weight_walk: launch shape not walkable");
  const int64_t out[EASYSPEC_WALK_FIELDS] = {p.grid, p.nw, p.TP, p.R, p.NB, w.w_max, w.w_pieces, w.w_out_of_range, w.x_max,
                                             w.x_slot_elems, w.x_out_of_range, w.tiles, w.missed_tiles, w.repeated_tiles,
                                             w.reread_tiles, w.uncovered_pieces};
  memcpy(report, out, sizeof out);
  return EASYSPEC_OK;
}

extern "C" int64_t easyspec_step_bytes(const easyspec_ctx* ctx) {
  if (!ctx) return 0;
  const Shape& s = ctx->s;
  const int64_t e = (int64_t)esize(s);
  const int64_t per_layer = ((int64_t)s.RQKV * s.d + (int64_t)s.d * s.HQ + 3ll * s.F * s.d) * e;
  int64_t bytes = per_layer * s.L + (int64_t)s.V * s.d * e;
  for (int b = 0; b < s.B; ++b)
    if (ctx->precise[b] > 0) bytes += (int64_t)(ctx->precise[b] + ctx->fuzzy[b] + 1) * s.L * 2 * s.Hkv * s.hd * e;
  return bytes;
}
