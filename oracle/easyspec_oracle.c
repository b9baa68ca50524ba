/*
 * EasySpec CPU oracle.  TEST INFRASTRUCTURE ONLY: a plain, slow, double-precision
 * implementation of the draft model's layer-sequential step (paper Alg. 1), the
 * layer-parallel fuzzy step (paper Alg. 2), bonus calibration (paper Sec. 3.2), greedy
 * acceptance (paper Alg. 3 at temperature 0) and acceptance by speculative sampling (Alg. 3,
 * Sec. 2.1) with the random numbers passed in, and the fuzzy step over one level of a token
 * tree (App. C).  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it; it shares no code with the HIP library.
 *
 * Arithmetic: every vector and accumulator is a double.  Parameters are read from the
 * caller's arrays (float32, or bf16 bit patterns widened on the fly).  The paper fixes no
 * precision, so where a bf16 model rounds is a reading, and the oracle keeps the readings apart
 * in two switches of the model (eso_model_set_rounding):
 *   kv_bf16   1: the KV cache holds bf16 values; 0: float32 values.
 *   act_mode  how a vector that enters a weight contraction (normalised hidden state,
 *             attention output, SiLU(gate)*up) is carried:
 *     ESO_ACT_PLAIN   not rounded at all; RMSNorm evaluated as written below, then contracted.
 *                     This is the plain reference the required tolerance of a bf16 model
 *                     (rel-L2 2e-2) refers to; it knows nothing of any kernel's operand format.
 *     ESO_ACT_SINGLE  rounded to one bf16 number (the normalised vector itself is rounded).
 *     ESO_ACT_PAIR    rounded to the sum of two bf16 numbers, hi = bf16(x) and lo = bf16(x - hi)
 *                     (about 16 significant bits), and RMSNorm enters a contraction in two
 *                     parts: the vector x*g (rounded) and the scalar rsqrt(mean(x^2)+eps), which
 *                     multiplies the contraction's result.  Without rounding this is the same
 *                     function; with it, it is the operand format of the HIP library, kept so
 *                     that a comparison can be ten times tighter than the bf16 noise floor.
 * Defaults: a bf16 model (cfg.bf16 == 1) starts with kv_bf16 = 1 and ESO_ACT_PAIR, a float32
 * model with kv_bf16 = 0 and ESO_ACT_PLAIN.
 *
 * Model function (pre-norm decoder; the paper names only the attention and MLP layers
 * and the normalisation before attention, App. E.1; the rest follows the benchmark shapes):
 *   RMSNorm(x; g) = x * rsqrt(mean(x^2) + eps) * g
 *   Attn_i(h) at position p = Wo * GQA(RoPE(Wq n + bq, p), K-cache incl. RoPE(Wk n + bk, p),
 *                                      V-cache incl. Wv n + bv),  n = RMSNorm(h; g_attn_i)
 *   MLP_i(h)  = Wd (SiLU(Wg y) * (Wu y)),  y = RMSNorm(h; g_mlp_i)
 *   logits    = Wlm RMSNorm(h_L; g_final)
 *
 * Parity pins (tests/test_oracle_*.py): sequential step against an independent library
 * decoder; Alg. 2 with all sets of size one == Alg. 1 bit for bit; calibration == token by
 * token sequential decoding bit for bit; greedy speculative decoding == vanilla greedy
 * decoding; speculative sampling reproduces the target distribution (exact integration over
 * the random inputs on tiny vocabularies) and reduces to greedy acceptance for one-hot
 * distributions; every root-to-node path of a token tree == chain drafting of that path, bit
 * for bit; the two-term bf16 rounding against a library's bf16 cast, its error bound and
 * planted mistakes; the three activation-rounding modes against the library decoder in double
 * precision on bf16 weights (plain equal, pair within 1e-4, single a hundred times further).
 * The numeric value of a fuzzy step with sets larger than one is fixed by no
 * number in the paper (its similarity table needs trained weights): that part is pinned
 * by a second composition of the same library blocks and by structural invariants only.
 *
 * OpenMP splits output rows only, so results do not depend on the thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  int32_t qkv_bias; /* 1: bq, bk, bv present */
  int32_t bf16;     /* 1: matrices are bf16 bit patterns and the bf16 rounding points apply */
  int32_t max_ctx;  /* KV slots per layer */
  double rms_eps, rope_theta;
} eso_config;

typedef struct {
  const void *wq, *wk, *wv, *wo, *wg, *wu, *wd; /* row-major [out][in], model dtype */
  const float *bq, *bk, *bv;                    /* NULL without bias */
  const float *g_attn, *g_mlp;
} eso_layer;

#define ESO_ACT_PLAIN 0
#define ESO_ACT_SINGLE 1
#define ESO_ACT_PAIR 2

typedef struct {
  eso_config cfg;
  eso_layer *layers;
  const void *embed, *lm_head; /* [vocab][d_model] */
  const float *g_final;
  int32_t act_mode; /* ESO_ACT_*: rounding of the vectors that enter a weight contraction */
  int32_t kv_bf16;  /* 1: cache entries are rounded to bf16 */
} eso_model;

#define ESO_MAX_TREE 64 /* nodes of one token tree */

typedef struct {
  const eso_model *m;
  float *K, *V; /* [layer][kv_head][slot][head_dim] */
  int32_t precise; /* slots [0, precise) hold values written by calibration */
  int32_t fuzzy;   /* slots [precise, precise+fuzzy) hold values written by fuzzy steps */
  double *attn_tap; /* optional [n_layers][d_model]: Attnoutput_i of the last single-token step */
  /* token tree (App. C): when n_tree > 0 the fuzzy slots are the nodes of a tree, node t in
   * slot precise + t, with its parent node (-1: child of the last precise token) and depth */
  int32_t n_tree;
  int32_t tree_parent[ESO_MAX_TREE], tree_depth[ESO_MAX_TREE];
  /* 0: layer-parallel attention only (Alg. 2).  1: full-layer parallel (the ablation of App. B):
   * every layer of a set, attention AND MLP, works from the set's input h_1, and the set's
   * output is h_1 plus the sum of what each layer adds:
   *   a_i = Attn_i(h_1),  m_i = MLP_i(h_1 + a_i),  h_out = h_1 + sum_i (a_i + m_i).
   * The paper names the variant without defining it; this is the reading "each layer of the set
   * runs whole, on its own device, from the same input".  With sets of one layer it is Alg. 1. */
  int32_t full_layer;
} eso_seq;

/* ---------------------------------------------------------------- storage formats */

static float bf16_bits_to_float(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

/* Round to the nearest bf16 value, ties to even (finite inputs). */
double eso_bf16_round(double x) {
  float f = (float)x;
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7FFFu + ((u >> 16) & 1u);
  u &= 0xFFFF0000u;
  memcpy(&f, &u, 4);
  return (double)f;
}

static double weight_at(const void *w, int bf16, size_t idx) {
  return bf16 ? (double)bf16_bits_to_float(((const uint16_t *)w)[idx]) : (double)((const float *)w)[idx];
}

/* x as the sum of two bf16 numbers: hi = bf16(x), lo = bf16(x - hi), both round-to-nearest-even
 * of a float32 (x is brought to float32 first, the type the vectors have before they are stored) */
double eso_bf16_pair_round(double x) {
  float xf = (float)x;
  double hi = eso_bf16_round((double)xf);
  double lo = eso_bf16_round((double)xf - hi);
  return hi + lo;
}

static double act_round(const eso_model *m, double x) {
  if (m->act_mode == ESO_ACT_PAIR) return eso_bf16_pair_round(x);
  if (m->act_mode == ESO_ACT_SINGLE) return eso_bf16_round(x);
  return x;
}
static float kv_store(const eso_model *m, double x) { return m->kv_bf16 ? (float)eso_bf16_round(x) : (float)x; }

/* ---------------------------------------------------------------- primitives */

/* y[r] = scale * sum_j W[r][j] x[j] (+ b[r]) */
void eso_matvec(const void *w, int bf16, const float *bias, double scale, int rows, int cols, const double *x,
                double *y) {
#pragma omp parallel for schedule(static)
  for (int r = 0; r < rows; ++r) {
    double acc = 0.0;
    size_t base = (size_t)r * (size_t)cols;
    for (int j = 0; j < cols; ++j) acc += weight_at(w, bf16, base + (size_t)j) * x[j];
    acc *= scale;
    y[r] = bias ? acc + (double)bias[r] : acc;
  }
}

/* RMSNorm(x; g) = x * rsqrt(mean(x^2) + eps) * g, returned in two parts:
 * xg[j] = x[j] * g[j] and the scalar rsqrt(mean(x^2) + eps). */
double eso_rmsnorm_split(const double *x, const float *g, int n, double eps, double *xg) {
  double ss = 0.0;
  for (int j = 0; j < n; ++j) ss += x[j] * x[j];
  for (int j = 0; j < n; ++j) xg[j] = x[j] * (double)g[j];
  return 1.0 / sqrt(ss / (double)n + eps);
}

/* RMSNorm(x; g) as written: the normalised vector times the gain */
void eso_rmsnorm(const double *x, const float *g, int n, double eps, double *y) {
  double ss = 0.0;
  for (int j = 0; j < n; ++j) ss += x[j] * x[j];
  double r = 1.0 / sqrt(ss / (double)n + eps);
  for (int j = 0; j < n; ++j) y[j] = (x[j] * r) * (double)g[j];
}

/* Rotary embedding of one head vector at position pos: element i pairs with i + hd/2,
 * angle = pos * theta^(-2i/hd). */
void eso_rope(double *x, int hd, int pos, double theta) {
  int half = hd / 2;
  for (int i = 0; i < half; ++i) {
    double ang = (double)pos * pow(theta, -2.0 * (double)i / (double)hd);
    double c = cos(ang), s = sin(ang);
    double a = x[i], b = x[i + half];
    x[i] = a * c - b * s;
    x[i + half] = b * c + a * s;
  }
}

double eso_silu(double z) { return z / (1.0 + exp(-z)); }

/* in-place softmax over n scores */
void eso_softmax(double *s, int n) {
  double mx = s[0];
  for (int t = 1; t < n; ++t)
    if (s[t] > mx) mx = s[t];
  double sum = 0.0;
  for (int t = 0; t < n; ++t) {
    s[t] = exp(s[t] - mx);
    sum += s[t];
  }
  for (int t = 0; t < n; ++t) s[t] /= sum;
}

/* index of the largest entry, lowest index on ties; optionally the gap to the runner-up */
int32_t eso_argmax(const double *x, int n, double *margin) {
  int best = 0;
  for (int j = 1; j < n; ++j)
    if (x[j] > x[best]) best = j;
  if (margin) {
    double second = -INFINITY;
    for (int j = 0; j < n; ++j)
      if (j != best && x[j] > second) second = x[j];
    *margin = x[best] - second;
  }
  return best;
}

/* RMSNorm(x; g) of a hidden state as the operand of a weight contraction, rounded as the model's
 * act_mode says.  Returns the factor that the contraction's result is to be multiplied by: 1, or
 * rsqrt(mean(x^2) + eps) when the norm is carried in two parts (ESO_ACT_PAIR). */
static double norm_operand(const eso_model *m, const double *x, const float *g, double *out) {
  int n = m->cfg.d_model;
  if (m->act_mode == ESO_ACT_PAIR) {
    double rs = eso_rmsnorm_split(x, g, n, m->cfg.rms_eps, out);
    for (int j = 0; j < n; ++j) out[j] = eso_bf16_pair_round(out[j]);
    return rs;
  }
  eso_rmsnorm(x, g, n, m->cfg.rms_eps, out);
  for (int j = 0; j < n; ++j) out[j] = act_round(m, out[j]);
  return 1.0;
}

/* ---------------------------------------------------------------- model / sequence objects */

eso_model *eso_model_create(const eso_config *cfg) {
  if (!cfg || cfg->n_layers < 1 || cfg->n_q_heads % cfg->n_kv_heads || cfg->head_dim % 2) return NULL;
  eso_model *m = (eso_model *)calloc(1, sizeof(eso_model));
  m->cfg = *cfg;
  m->layers = (eso_layer *)calloc((size_t)cfg->n_layers, sizeof(eso_layer));
  m->act_mode = cfg->bf16 ? ESO_ACT_PAIR : ESO_ACT_PLAIN;
  m->kv_bf16 = cfg->bf16 ? 1 : 0;
  return m;
}

/* Where the model rounds (see the head of this file).  Returns 0, or -1 for an unknown mode. */
int eso_model_set_rounding(eso_model *m, int32_t act_mode, int32_t kv_bf16) {
  if (!m || act_mode < ESO_ACT_PLAIN || act_mode > ESO_ACT_PAIR) return -1;
  m->act_mode = act_mode;
  m->kv_bf16 = kv_bf16 ? 1 : 0;
  return 0;
}

void eso_model_set_layer(eso_model *m, int i, const void *wq, const void *wk, const void *wv, const void *wo,
                         const void *wg, const void *wu, const void *wd, const float *bq, const float *bk,
                         const float *bv, const float *g_attn, const float *g_mlp) {
  eso_layer *l = &m->layers[i];
  l->wq = wq; l->wk = wk; l->wv = wv; l->wo = wo; l->wg = wg; l->wu = wu; l->wd = wd;
  l->bq = bq; l->bk = bk; l->bv = bv; l->g_attn = g_attn; l->g_mlp = g_mlp;
}

void eso_model_set_top(eso_model *m, const void *embed, const float *g_final, const void *lm_head) {
  m->embed = embed; m->g_final = g_final; m->lm_head = lm_head;
}

void eso_model_destroy(eso_model *m) {
  if (!m) return;
  free(m->layers);
  free(m);
}

static size_t kv_elems(const eso_config *c) {
  return (size_t)c->n_layers * (size_t)c->n_kv_heads * (size_t)c->max_ctx * (size_t)c->head_dim;
}

eso_seq *eso_seq_create(const eso_model *m) {
  eso_seq *s = (eso_seq *)calloc(1, sizeof(eso_seq));
  s->m = m;
  s->K = (float *)calloc(kv_elems(&m->cfg), sizeof(float));
  s->V = (float *)calloc(kv_elems(&m->cfg), sizeof(float));
  return s;
}

void eso_seq_destroy(eso_seq *s) {
  if (!s) return;
  free(s->K); free(s->V); free(s->attn_tap); free(s);
}

float *eso_seq_k(eso_seq *s) { return s->K; }
float *eso_seq_v(eso_seq *s) { return s->V; }
int32_t eso_seq_precise(const eso_seq *s) { return s->precise; }
int32_t eso_seq_fuzzy(const eso_seq *s) { return s->fuzzy; }
void eso_seq_set_full_layer(eso_seq *s, int32_t on) { s->full_layer = on ? 1 : 0; }
void eso_seq_set_lens(eso_seq *s, int32_t precise, int32_t fuzzy) { s->precise = precise; s->fuzzy = fuzzy; s->n_tree = 0; }
double *eso_seq_enable_attn_tap(eso_seq *s) {
  if (!s->attn_tap) s->attn_tap = (double *)calloc((size_t)s->m->cfg.n_layers * (size_t)s->m->cfg.d_model, sizeof(double));
  return s->attn_tap;
}

static float *kv_row(const eso_seq *s, float *base, int layer, int kvh, int slot) {
  const eso_config *c = &s->m->cfg;
  return base + (((size_t)layer * c->n_kv_heads + kvh) * (size_t)c->max_ctx + (size_t)slot) * (size_t)c->head_dim;
}

/* ---------------------------------------------------------------- the three blocks */

/* Attnoutput = Attn_layer(h) for a token whose rotary position is rpos; stores that token's
 * k, v in cache slot `slot` (values computed from THIS h, whatever h is) and attends to the
 * n_vis slots vis[0] < vis[1] < ... (which include `slot`); vis == NULL means slots 0..slot. */
static void attn_block_vis(eso_seq *s, int layer, const double *h, int slot, int rpos, const int32_t *vis, int n_vis,
                           double *out) {
  const eso_config *c = &s->m->cfg;
  const eso_layer *l = &s->m->layers[layer];
  int d = c->d_model, hd = c->head_dim, nq = c->n_q_heads, nkv = c->n_kv_heads, grp = nq / nkv;
  double *n = (double *)malloc(sizeof(double) * (size_t)d);
  double *q = (double *)malloc(sizeof(double) * (size_t)nq * hd);
  double *k = (double *)malloc(sizeof(double) * (size_t)nkv * hd);
  double *v = (double *)malloc(sizeof(double) * (size_t)nkv * hd);
  double *o = (double *)malloc(sizeof(double) * (size_t)nq * hd);
  const int nv = vis ? n_vis : slot + 1;
  double *scores = (double *)malloc(sizeof(double) * (size_t)nq * (size_t)nv);

  double rs = norm_operand(s->m, h, l->g_attn, n);
  eso_matvec(l->wq, c->bf16, l->bq, rs, nq * hd, d, n, q);
  eso_matvec(l->wk, c->bf16, l->bk, rs, nkv * hd, d, n, k);
  eso_matvec(l->wv, c->bf16, l->bv, rs, nkv * hd, d, n, v);
  for (int a = 0; a < nq; ++a) eso_rope(q + (size_t)a * hd, hd, rpos, c->rope_theta);
  for (int g = 0; g < nkv; ++g) {
    eso_rope(k + (size_t)g * hd, hd, rpos, c->rope_theta);
    float *kr = kv_row(s, s->K, layer, g, slot), *vr = kv_row(s, s->V, layer, g, slot);
    for (int e = 0; e < hd; ++e) {
      kr[e] = kv_store(s->m, k[(size_t)g * hd + e]);
      vr[e] = kv_store(s->m, v[(size_t)g * hd + e]);
    }
  }
  double scale = 1.0 / sqrt((double)hd);
#pragma omp parallel for schedule(static)
  for (int a = 0; a < nq; ++a) { /* heads are independent; each uses its own score row */
    int g = a / grp; /* query head a reads KV head a / (Hq/Hkv) */
    const double *qa = q + (size_t)a * hd;
    double *sc = scores + (size_t)a * (size_t)nv;
    for (int t = 0; t < nv; ++t) {
      const float *kr = kv_row(s, s->K, layer, g, vis ? vis[t] : t);
      double dot = 0.0;
      for (int e = 0; e < hd; ++e) dot += qa[e] * (double)kr[e];
      sc[t] = dot * scale;
    }
    eso_softmax(sc, nv);
    for (int e = 0; e < hd; ++e) {
      double acc = 0.0;
      for (int t = 0; t < nv; ++t) acc += sc[t] * (double)kv_row(s, s->V, layer, g, vis ? vis[t] : t)[e];
      o[(size_t)a * hd + e] = act_round(s->m, acc);
    }
  }
  eso_matvec(l->wo, c->bf16, NULL, 1.0, d, nq * hd, o, out);
  free(n); free(q); free(k); free(v); free(o); free(scores);
}

/* the causal case: the token at position pos sits in slot pos and attends to slots 0..pos */
static void attn_block(eso_seq *s, int layer, const double *h, int pos, double *out) {
  attn_block_vis(s, layer, h, pos, pos, NULL, 0, out);
}

/* MLPoutput = MLP_layer(h) */
static void mlp_block(const eso_model *m, int layer, const double *h, double *out) {
  const eso_config *c = &m->cfg;
  const eso_layer *l = &m->layers[layer];
  int d = c->d_model, f = c->d_ffn;
  double *y = (double *)malloc(sizeof(double) * (size_t)d);
  double *g = (double *)malloc(sizeof(double) * (size_t)f);
  double *u = (double *)malloc(sizeof(double) * (size_t)f);
  double rs = norm_operand(m, h, l->g_mlp, y);
  eso_matvec(l->wg, c->bf16, NULL, rs, f, d, y, g);
  eso_matvec(l->wu, c->bf16, NULL, rs, f, d, y, u);
  for (int j = 0; j < f; ++j) g[j] = act_round(m, eso_silu(g[j]) * u[j]);
  eso_matvec(l->wd, c->bf16, NULL, 1.0, d, f, g, out);
  free(y); free(g); free(u);
}

static void embed_row(const eso_model *m, int32_t token, double *h) {
  int d = m->cfg.d_model;
  for (int j = 0; j < d; ++j) h[j] = weight_at(m->embed, m->cfg.bf16, (size_t)token * d + j);
}

static void head(const eso_model *m, const double *h, double *logits) {
  const eso_config *c = &m->cfg;
  double *x = (double *)malloc(sizeof(double) * (size_t)c->d_model);
  double rs = norm_operand(m, h, m->g_final, x);
  eso_matvec(m->lm_head, c->bf16, NULL, rs, c->vocab, c->d_model, x, logits);
  free(x);
}

/* ---------------------------------------------------------------- paper Alg. 1 */

/* One layer-sequential forward of one token at position precise (requires fuzzy == 0);
 * the slot it writes is precise.  Returns 0, or -1 on a bad state. */
int eso_sequential_step(eso_seq *s, int32_t token, double *logits, double *hidden_out) {
  const eso_config *c = &s->m->cfg;
  if (s->fuzzy != 0 || s->precise + 1 > c->max_ctx || token < 0 || token >= c->vocab) return -1;
  int d = c->d_model, pos = s->precise;
  double *h = (double *)malloc(sizeof(double) * (size_t)d), *a = (double *)malloc(sizeof(double) * (size_t)d);
  double *mo = (double *)malloc(sizeof(double) * (size_t)d);
  embed_row(s->m, token, h);
  for (int i = 0; i < c->n_layers; ++i) {
    attn_block(s, i, h, pos, a);                       /* attention of layer i on the running residual */
    if (s->attn_tap) memcpy(s->attn_tap + (size_t)i * d, a, sizeof(double) * (size_t)d);
    for (int j = 0; j < d; ++j) h[j] = h[j] + a[j];    /* residual update after attention */
    mlp_block(s->m, i, h, mo);                         /* MLP of layer i on the updated residual */
    for (int j = 0; j < d; ++j) h[j] = h[j] + mo[j];   /* residual update after the MLP: input of layer i+1 */
  }
  if (hidden_out) memcpy(hidden_out, h, sizeof(double) * (size_t)d);
  if (logits) head(s->m, h, logits);
  s->precise += 1;
  free(h); free(a); free(mo);
  return 0;
}

/* Full-layer parallel set (the ablation of App. B; see eso_seq.full_layer): with the Attnoutputs
 * a[i] = Attn_i(h_1) of the set [lo, hi) known, every MLP reads h_1 plus its own layer's
 * Attnoutput, and all contributions are added to h_1.  On entry h == h1.  mo: scratch. */
static void full_layer_set(const eso_seq *s, int lo, int hi, const double *h1, const double *a, double *h, double *mo) {
  const int d = s->m->cfg.d_model;
  double *t = (double *)malloc(sizeof(double) * (size_t)d);
  for (int i = lo; i < hi; ++i) {
    const double *ai = a + (size_t)i * d;
    for (int e = 0; e < d; ++e) t[e] = h1[e] + ai[e];          /* this layer's own h' = h_1 + Attnoutput_i */
    mlp_block(s->m, i, t, mo);                                  /* MLP_i(h_1 + Attnoutput_i) */
    for (int e = 0; e < d; ++e) h[e] = (h[e] + ai[e]) + mo[e];  /* h_out = h_1 + sum_i (a_i + m_i), added in layer order */
  }
  free(t);
}

/* ---------------------------------------------------------------- paper Alg. 2 */

/* One layer-parallel fuzzy forward of one token.  bounds[0]=0 < ... < bounds[n_sets]=L;
 * set j = layers [bounds[j], bounds[j+1]).  Every attention layer of a set reads the hidden
 * state that enters the set; the MLPs stay sequential.  Writes slot precise+fuzzy in every
 * layer and counts it as fuzzy. */
int eso_fuzzy_step(eso_seq *s, const int32_t *bounds, int32_t n_sets, int32_t token, double *logits,
                   double *hidden_out) {
  const eso_config *c = &s->m->cfg;
  if (n_sets < 1 || bounds[0] != 0 || bounds[n_sets] != c->n_layers) return -1;
  for (int j = 0; j < n_sets; ++j)
    if (bounds[j + 1] <= bounds[j]) return -1;
  if (s->precise + s->fuzzy + 1 > c->max_ctx || token < 0 || token >= c->vocab || s->n_tree != 0) return -1;
  int d = c->d_model, pos = s->precise + s->fuzzy;
  double *h = (double *)malloc(sizeof(double) * (size_t)d), *h1 = (double *)malloc(sizeof(double) * (size_t)d);
  double *a = (double *)malloc(sizeof(double) * (size_t)d * (size_t)c->n_layers);
  double *mo = (double *)malloc(sizeof(double) * (size_t)d);
  embed_row(s->m, token, h);
  for (int j = 0; j < n_sets; ++j) {
    int lo = bounds[j], hi = bounds[j + 1];
    memcpy(h1, h, sizeof(double) * (size_t)d);                                 /* the state that enters the set */
    for (int i = lo; i < hi; ++i) attn_block(s, i, h1, pos, a + (size_t)i * d); /* every attention layer of the set reads it */
    if (s->full_layer) {
      full_layer_set(s, lo, hi, h1, a, h, mo); /* App. B ablation */
    } else {
      for (int i = lo; i < hi; ++i) {
        const double *ai = a + (size_t)i * d;
        for (int e = 0; e < d; ++e) h[e] = h[e] + ai[e];  /* add layer i's parked attention output */
        mlp_block(s->m, i, h, mo);                        /* its MLP sees the running residual: the MLPs stay in layer order */
        for (int e = 0; e < d; ++e) h[e] = h[e] + mo[e];
      }
    }
  }
  if (s->attn_tap) memcpy(s->attn_tap, a, sizeof(double) * (size_t)d * (size_t)c->n_layers);
  if (hidden_out) memcpy(hidden_out, h, sizeof(double) * (size_t)d);
  if (logits) head(s->m, h, logits);
  s->fuzzy += 1;
  free(h); free(h1); free(a); free(mo);
  return 0;
}

/* ---------------------------------------------------------------- token tree (App. C) */

/* One layer-parallel fuzzy forward (Alg. 2) of the n tokens of one tree level.  Node j is the
 * child of node parents[j] of the tree drafted so far (an index below the node count before
 * this call), or of the last precise token (-1).  It takes the next free slot, its rotary
 * position is precise + depth (the position it would have in its own root-to-node sequence),
 * and it attends to the precise slots, its ancestors and itself: the row of the 2-D tree mask.
 * The nodes of a level do not see each other, so each is one Alg. 2 forward of its own.
 * Needs fuzzy == node count (no chain-drafted slots in between).  logits: [n][vocab] or NULL;
 * hidden_out: [n][d_model] or NULL. */
int eso_fuzzy_tree_step(eso_seq *s, const int32_t *bounds, int32_t n_sets, int32_t n, const int32_t *tokens,
                        const int32_t *parents, double *logits, double *hidden_out) {
  const eso_config *c = &s->m->cfg;
  if (n_sets < 1 || bounds[0] != 0 || bounds[n_sets] != c->n_layers) return -1;
  for (int j = 0; j < n_sets; ++j)
    if (bounds[j + 1] <= bounds[j]) return -1;
  if (n < 1 || s->fuzzy != s->n_tree || s->n_tree + n > ESO_MAX_TREE || s->precise + s->fuzzy + n > c->max_ctx) return -1;
  for (int j = 0; j < n; ++j)
    if (tokens[j] < 0 || tokens[j] >= c->vocab || parents[j] < -1 || parents[j] >= s->n_tree) return -1;
  int d = c->d_model, P = s->precise, f = s->n_tree;
  double *h = (double *)malloc(sizeof(double) * (size_t)d), *h1 = (double *)malloc(sizeof(double) * (size_t)d);
  double *a = (double *)malloc(sizeof(double) * (size_t)d * (size_t)c->n_layers);
  double *mo = (double *)malloc(sizeof(double) * (size_t)d);
  int32_t *vis = (int32_t *)malloc(sizeof(int32_t) * (size_t)(P + ESO_MAX_TREE + 1));
  for (int j = 0; j < n; ++j) {
    const int node = f + j, slot = P + node;
    const int depth = parents[j] < 0 ? 0 : s->tree_depth[parents[j]] + 1;
    /* visible slots in ascending order: precise prefix, ancestors (root first), the node itself */
    int nv = 0;
    for (int t = 0; t < P; ++t) vis[nv++] = t;
    int chain[ESO_MAX_TREE], nc = 0;
    for (int t = parents[j]; t >= 0; t = s->tree_parent[t]) chain[nc++] = t;
    for (int t = nc - 1; t >= 0; --t) vis[nv++] = P + chain[t]; /* a parent always has a lower index than its child */
    vis[nv++] = slot;
    embed_row(s->m, tokens[j], h);
    for (int g = 0; g < n_sets; ++g) {
      int lo = bounds[g], hi = bounds[g + 1];
      memcpy(h1, h, sizeof(double) * (size_t)d);                                                      /* the state that enters the set */
      for (int i = lo; i < hi; ++i) attn_block_vis(s, i, h1, slot, P + depth, vis, nv, a + (size_t)i * d);
      if (s->full_layer) {
        full_layer_set(s, lo, hi, h1, a, h, mo); /* App. B ablation */
      } else {
        for (int i = lo; i < hi; ++i) {
          const double *ai = a + (size_t)i * d;
          for (int e = 0; e < d; ++e) h[e] = h[e] + ai[e];  /* as in eso_fuzzy_step: parked attention output, */
          mlp_block(s->m, i, h, mo);                        /* then the MLP on the running residual */
          for (int e = 0; e < d; ++e) h[e] = h[e] + mo[e];
        }
      }
    }
    if (hidden_out) memcpy(hidden_out + (size_t)j * d, h, sizeof(double) * (size_t)d);
    if (logits) head(s->m, h, logits + (size_t)j * c->vocab);
    s->tree_parent[node] = parents[j];
    s->tree_depth[node] = depth;
  }
  s->n_tree += n;
  s->fuzzy += n;
  free(h); free(h1); free(a); free(mo); free(vis);
  return 0;
}

/* ---------------------------------------------------------------- bonus calibration (Sec. 3.2) */

/* Drop every fuzzy slot, then run ONE token-parallel, layer-sequential forward over the
 * n tokens (accepted tokens followed by the bonus token) at positions precise..precise+n-1.
 * Their k, v overwrite those slots and count as precise.  logits_all: [n][vocab] or NULL;
 * hidden_all: [n][d_model] or NULL.  The last row's logits give the next draft token. */
int eso_calibrate(eso_seq *s, const int32_t *tokens, int32_t n, double *logits_all, double *hidden_all) {
  const eso_config *c = &s->m->cfg;
  if (n < 1 || s->precise + n > c->max_ctx) return -1;
  for (int r = 0; r < n; ++r)
    if (tokens[r] < 0 || tokens[r] >= c->vocab) return -1;
  s->fuzzy = 0;
  s->n_tree = 0;
  int d = c->d_model, p0 = s->precise;
  double *H = (double *)malloc(sizeof(double) * (size_t)n * d);
  double *a = (double *)malloc(sizeof(double) * (size_t)d), *mo = (double *)malloc(sizeof(double) * (size_t)d);
  for (int r = 0; r < n; ++r) embed_row(s->m, tokens[r], H + (size_t)r * d);
  for (int i = 0; i < c->n_layers; ++i) {
    /* rows in increasing position: row r stores its k, v before it attends, so it sees rows <= r */
    for (int r = 0; r < n; ++r) {
      double *h = H + (size_t)r * d;
      attn_block(s, i, h, p0 + r, a);
      for (int e = 0; e < d; ++e) h[e] = h[e] + a[e];
    }
    for (int r = 0; r < n; ++r) {
      double *h = H + (size_t)r * d;
      mlp_block(s->m, i, h, mo);
      for (int e = 0; e < d; ++e) h[e] = h[e] + mo[e];
    }
  }
  if (hidden_all) memcpy(hidden_all, H, sizeof(double) * (size_t)n * d);
  if (logits_all)
    for (int r = 0; r < n; ++r) head(s->m, H + (size_t)r * d, logits_all + (size_t)r * c->vocab);
  s->precise += n;
  free(H); free(a); free(mo);
  return 0;
}

/* Logits of the last calibrated row only (what a drafter needs): same forward as
 * eso_calibrate but the head runs on one row. */
int eso_calibrate_last(eso_seq *s, const int32_t *tokens, int32_t n, double *logits_last) {
  const eso_config *c = &s->m->cfg;
  double *hid = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1) * c->d_model);
  int rc = eso_calibrate(s, tokens, n, NULL, hid);
  if (rc == 0 && logits_last) head(s->m, hid + (size_t)(n - 1) * c->d_model, logits_last);
  free(hid);
  return rc;
}

/* ---------------------------------------------------------------- Alg. 3 at temperature 0 */

/* With one-hot draft and target distributions a drafted token is accepted exactly when it
 * equals the target model's argmax at that position; the bonus token is the target's argmax
 * at the first rejected position, or at position gamma when everything was accepted.
 * draft: [gamma]; target: [gamma+1]. */
void eso_greedy_accept(const int32_t *draft, const int32_t *target, int32_t gamma, int32_t *accept_len,
                       int32_t *bonus) {
  int m = 0;
  while (m < gamma && draft[m] == target[m]) ++m;
  *accept_len = m;
  *bonus = target[m];
}

/* Acceptance by speculative sampling (Alg. 3; bonus distribution of Sec. 2.1) for one
 * sequence, with the random numbers given: r[i] in [0,1) decides position i, u in [0,1)
 * draws the bonus token.
 *   p'_i = softmax(draft_logits[i] / T), i < gamma;  p_i = softmax(target_logits[i] / T), i <= gamma.
 *   Position i is rejected when r_i > p_i(x'_i) / p'_i(x'_i), evaluated as r_i * p'_i(x'_i) > p_i(x'_i)
 *   (same decision, no division by a vanishing probability); m = index of the first rejection,
 *   or gamma.
 *   Bonus distribution: q = max(0, p_m - p'_m) if m < gamma (the printed algorithm's index is
 *   garbled; this is the equation of Sec. 2.1: the distributions at the first rejected
 *   position), else q = p_gamma.  Normalisation and draw together: bonus = the lowest v whose
 *   running sum q(0) + ... + q(v) exceeds u * sum(q).  If the residual is identically zero
 *   (p_m == p'_m, where a rejection cannot happen for r < 1) q falls back to p_m.
 * margin (optional): the smallest relative distance of any decision taken from its threshold,
 * so that a comparison with another implementation can set aside decisions that rounding
 * could flip. */
static void softmax_t(const float *logits, int32_t V, double T, double *p) {
  double mx = -INFINITY;
  for (int v = 0; v < V; ++v) if ((double)logits[v] > mx) mx = (double)logits[v];
  double z = 0.0;
  for (int v = 0; v < V; ++v) { p[v] = exp(((double)logits[v] - mx) / T); z += p[v]; }
  for (int v = 0; v < V; ++v) p[v] /= z;
}

int eso_accept(const int32_t *draft, const float *draft_logits, const float *target_logits, const float *r, float u,
               int32_t gamma, int32_t V, double T, int32_t *accept_len, int32_t *bonus, double *margin) {
  if (gamma < 0 || V < 1 || !(T > 0.0)) return -1;
  double *p = (double *)malloc(sizeof(double) * (size_t)V), *pd = (double *)malloc(sizeof(double) * (size_t)V);
  if (!p || !pd) { free(p); free(pd); return -1; }
  double mg = INFINITY;
  int m = 0;
  for (; m < gamma; ++m) {
    const int x = draft[m];
    if (x < 0 || x >= V) { free(p); free(pd); return -1; }
    softmax_t(target_logits + (size_t)m * V, V, T, p);
    softmax_t(draft_logits + (size_t)m * V, V, T, pd);
    const double lhs = (double)r[m] * pd[x], rhs = p[x];
    const double big = fmax(fabs(lhs), fabs(rhs));
    if (big > 0.0) mg = fmin(mg, fabs(lhs - rhs) / big);
    if (lhs > rhs) break; /* rejected; p and pd hold the distributions of this position */
  }
  if (m == gamma) {
    softmax_t(target_logits + (size_t)gamma * V, V, T, p);
  } else {
    double s = 0.0;
    for (int v = 0; v < V; ++v) { pd[v] = fmax(0.0, p[v] - pd[v]); s += pd[v]; }
    if (s > 0.0) memcpy(p, pd, sizeof(double) * (size_t)V);
  }
  double total = 0.0;
  for (int v = 0; v < V; ++v) total += p[v];
  const double thr = (double)u * total;
  double run = 0.0;
  int pick = -1, last_pos = 0;
  for (int v = 0; v < V; ++v) {
    if (p[v] > 0.0) last_pos = v;
    const double before = run;
    run += p[v];
    if (run > thr) {
      pick = v;
      const double up = run - thr, down = v == 0 ? INFINITY : thr - before; /* distances to the two neighbouring outcomes */
      mg = fmin(mg, fmin(up, down) / total);
      break;
    }
  }
  if (pick < 0) { pick = last_pos; mg = 0.0; }
  *accept_len = m;
  *bonus = pick;
  if (margin) *margin = mg;
  free(p);
  free(pd);
  return 0;
}

/* ---------------------------------------------------------------- layer-parallel strategy (Sec. 3.1.1) */

/* policy 0 ("aligned", the rule in the text): first and last layer alone; the layers between
 * are cut at multiples of N: 1..N-1, N..2N-1, ..., the last set stopping before layer L-1.
 * policy 1 ("packed", the 16-layer row of the strategy table): first and last layer alone;
 * sets of N consecutive layers starting at layer 1, the last one truncated before layer L-1.
 * bounds must hold L+1 entries.  Returns 0 or -1. */
int eso_default_groups(int32_t L, int32_t N, int32_t policy, int32_t *bounds, int32_t *n_sets) {
  if (L < 1 || N < 1 || (policy != 0 && policy != 1)) return -1;
  int n = 0;
  bounds[n++] = 0;
  if (L == 1) { bounds[n] = 1; *n_sets = 1; return 0; }
  bounds[n++] = 1; /* layer 0 alone */
  int last = L - 1; /* layer L-1 alone */
  int cur = 1;
  while (cur < last) {
    int next = (policy == 0) ? ((cur / N) + 1) * N : cur + N;
    if (next > last) next = last;
    bounds[n++] = next;
    cur = next;
  }
  bounds[n] = L;
  *n_sets = n;
  return 0;
}
