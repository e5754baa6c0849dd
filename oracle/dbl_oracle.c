/*
 * dbl_oracle.c -- plain, slow CPU oracle for the verify -> accept -> retrieve ->
 * commit path of Double (Double Retrieval Speculative Parallelism).
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call, link or import
 * this file.  It shares no code with the HIP library: every routine here is
 * written straight from the definition it cites, in fp64, one row at a time,
 * with no blocking, fusion or reordering.
 *
 * What each part follows (paper = arxiv 2601.05524):
 *   forward      Sec. 2.1 ("single parallel forward pass" of the target model
 *                over the drafted tokens) and App. D.2 (causal mask: every window
 *                position conditioned on the prefix and the window rows before
 *                it).  The paper uses stock LLaMA / Qwen3 decoders and prints no
 *                layer equations; the layer below is the standard pre-norm
 *                decoder: RMSNorm, GQA attention with rotary embedding (and
 *                Qwen3's per-head RMSNorm on q and k), SwiGLU MLP, LM head.
 *   greedy       App. D.2, greedy decoding: a draft survives iff it equals the
 *                target's top-1; the first mismatch is replaced by that top-1.
 *   sampling     Sec. 2.1: accept x_i with probability min(1, p(x_i)/q(x_i));
 *                on rejection draw from norm(max(0, p - q)); if every draft
 *                survives one extra token is drawn from the last row.
 *                Sec. 5.3 / App. D.2 (T > 0): guidance after a rejection is
 *                discarded.
 *   retrieve     Alg. 3 (descending n-gram loop, self-sequence search) and
 *                Eq. 2 (retrieve up to d continuation tokens).
 *   commit       Alg. 1 ("rollback"), Alg. 2 (truncate x, update datastore).
 *
 * Numerics for bf16 models (the paper only says "bf16"): weights hold bf16
 * values; all arithmetic is fp64; values are rounded to bf16 (nearest-even) at
 *   r1 the output of every RMSNorm that feeds a projection,
 *   r2 q and k after (qk-norm and) RoPE, and v, i.e. what the KV cache holds,
 *   (the softmax probabilities are NOT rounded: they weight v in full precision),
 *   r3 the attention output before the output projection,
 *   r4 silu(gate)*up before the down projection.
 * Logits are never rounded.  fp32 models have no rounding points.
 *
 * Parity status: every function here is pinned by tests/test_oracle_*.py
 * (closed forms, special cases reducing to library routines, brute force,
 * invariants).  Full-depth 70B / 32B logits are "parity unpinned" on the CPU
 * (too large to run); they are pinned through 2-layer full-width slices.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ config */

typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  int32_t qk_norm; /* 1: per-head RMSNorm on q and k (Qwen3) */
  int32_t dtype;   /* 0: fp32 model, 1: bf16 model (rounding points r1..r4) */
  int32_t max_ctx;
  double rms_eps, rope_base;
} orc_cfg;

enum {
  ORC_T_EMB = 0, ORC_T_LM = 1, ORC_T_GF = 2,
  ORC_T_G1 = 10, ORC_T_WQ = 11, ORC_T_WK = 12, ORC_T_WV = 13, ORC_T_GQ = 14,
  ORC_T_GK = 15, ORC_T_WO = 16, ORC_T_G2 = 17, ORC_T_WG = 18, ORC_T_WU = 19,
  ORC_T_WD = 20
};

typedef struct {
  float *g1, *wq, *wk, *wv, *gq, *gk, *wo, *g2, *wg, *wu, *wd;
} orc_layer;

typedef struct {
  orc_cfg cfg;
  float *emb, *lm, *gf;
  orc_layer *layers;
} orc_model;

typedef struct {
  const orc_model *model;
  int32_t kv_len;   /* committed KV slots */
  int32_t hist_len; /* committed tokens (prompt + generated) */
  int32_t max_hist;
  int32_t *hist;
  double *kc, *vc;  /* [layer][kv_head][max_ctx][head_dim] */
} orc_seq;

/* ----------------------------------------------------------- bf16 rounding */

/* Round a double to the nearest bf16 value (8 significant bits), ties to even.
 * Done on the fp64 value directly so that no intermediate fp32 rounding occurs.
 * Magnitudes met here are far from the bf16 overflow / subnormal ranges. */
double orc_round_bf16(double x) {
  if (x == 0.0 || !isfinite(x)) return x;
  int e;
  double m = frexp(x, &e);          /* |m| in [0.5, 1) */
  m = nearbyint(m * 256.0) / 256.0; /* default rounding mode: nearest even */
  return ldexp(m, e);
}

static double rnd(const orc_cfg *c, double x) {
  return c->dtype == 1 ? orc_round_bf16(x) : x;
}

/* --------------------------------------------------------- Philox4x32-10 */

/* Salmon et al., "Parallel random numbers: as easy as 1, 2, 3" (SC'11). */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int r = 0; r < 10; ++r) {
    uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Uniform in (0,1) from 23 random bits: ((x >> 9) + 0.5) * 2^-23. */
static double u01(uint32_t x) { return ((double)(x >> 9) + 0.5) * (1.0 / 8388608.0); }

/* ------------------------------------------------- synthetic model weights */

/* One weight = 0.02-std near-Gaussian from one Philox block: the sum of its
 * eight 16-bit halves (Irwin-Hall, exact integer), centred and scaled by one
 * fp32 constant, then (bf16 models) rounded to bf16.  Counter = (element index
 * low, high, tensor id, layer); key = seed.  Integer-only up to one fp32
 * multiply, so every implementation produces the same bits. */
float orc_weight_value(uint64_t seed, int tensor_id, int layer, uint64_t elem, int dtype) {
  uint32_t ctr[4] = {(uint32_t)elem, (uint32_t)(elem >> 32), (uint32_t)tensor_id, (uint32_t)layer};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t o[4];
  orc_philox4x32_10(ctr, key, o);
  int32_t s = 0;
  for (int i = 0; i < 4; ++i) s += (int32_t)(o[i] & 0xffffu) + (int32_t)(o[i] >> 16);
  /* var of one 16-bit uniform integer = (65536^2 - 1)/12 */
  const float c = (float)(0.02 / sqrt(8.0 * (65536.0 * 65536.0 - 1.0) / 12.0));
  float w = (float)(s - 262140) * c;
  if (dtype == 1) w = (float)orc_round_bf16((double)w);
  return w;
}

void orc_weight_fill(uint64_t seed, int tensor_id, int layer, uint64_t first, uint64_t n,
                     int dtype, float *out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < (int64_t)n; ++i)
    out[i] = orc_weight_value(seed, tensor_id, layer, first + (uint64_t)i, dtype);
}

static float *alloc_fill(uint64_t seed, int id, int layer, uint64_t n, int dtype) {
  float *p = (float *)malloc(sizeof(float) * (n ? n : 1));
  if (p) orc_weight_fill(seed, id, layer, 0, n, dtype, p);
  return p;
}

static float *alloc_ones(uint64_t n) {
  float *p = (float *)malloc(sizeof(float) * (n ? n : 1));
  if (p) for (uint64_t i = 0; i < n; ++i) p[i] = 1.0f;
  return p;
}

/* Matrices and embeddings ~ N(0, 0.02) from the seed; every norm gain = 1. */
orc_model *orc_model_new(const orc_cfg *cfg, uint64_t seed) {
  orc_model *m = (orc_model *)calloc(1, sizeof(orc_model));
  if (!m) return NULL;
  m->cfg = *cfg;
  const uint64_t d = cfg->d_model, hd = cfg->head_dim, V = cfg->vocab, F = cfg->d_ffn;
  const uint64_t nq = (uint64_t)cfg->n_q_heads * hd, nkv = (uint64_t)cfg->n_kv_heads * hd;
  const int dt = cfg->dtype;
  m->emb = alloc_fill(seed, ORC_T_EMB, 0, V * d, dt);
  m->lm = alloc_fill(seed, ORC_T_LM, 0, V * d, dt);
  m->gf = alloc_ones(d);
  m->layers = (orc_layer *)calloc(cfg->n_layers ? cfg->n_layers : 1, sizeof(orc_layer));
  for (int l = 0; l < cfg->n_layers; ++l) {
    orc_layer *L = &m->layers[l];
    L->g1 = alloc_ones(d);
    L->wq = alloc_fill(seed, ORC_T_WQ, l, nq * d, dt);
    L->wk = alloc_fill(seed, ORC_T_WK, l, nkv * d, dt);
    L->wv = alloc_fill(seed, ORC_T_WV, l, nkv * d, dt);
    L->gq = alloc_ones(hd);
    L->gk = alloc_ones(hd);
    L->wo = alloc_fill(seed, ORC_T_WO, l, d * nq, dt);
    L->g2 = alloc_ones(d);
    L->wg = alloc_fill(seed, ORC_T_WG, l, F * d, dt);
    L->wu = alloc_fill(seed, ORC_T_WU, l, F * d, dt);
    L->wd = alloc_fill(seed, ORC_T_WD, l, d * F, dt);
  }
  return m;
}

void orc_model_free(orc_model *m) {
  if (!m) return;
  for (int l = 0; l < m->cfg.n_layers; ++l) {
    orc_layer *L = &m->layers[l];
    free(L->g1); free(L->wq); free(L->wk); free(L->wv); free(L->gq); free(L->gk);
    free(L->wo); free(L->g2); free(L->wg); free(L->wu); free(L->wd);
  }
  free(m->layers); free(m->emb); free(m->lm); free(m->gf); free(m);
}

/* Row-major [out_features][in_features] storage of one tensor (tests read and
 * overwrite weights through this). */
float *orc_model_tensor(orc_model *m, int tensor_id, int layer, int64_t *n_elems) {
  const orc_cfg *c = &m->cfg;
  const int64_t d = c->d_model, hd = c->head_dim, V = c->vocab, F = c->d_ffn;
  const int64_t nq = (int64_t)c->n_q_heads * hd, nkv = (int64_t)c->n_kv_heads * hd;
  orc_layer *L = (layer >= 0 && layer < c->n_layers) ? &m->layers[layer] : NULL;
  float *p = NULL; int64_t n = 0;
  switch (tensor_id) {
    case ORC_T_EMB: p = m->emb; n = V * d; break;
    case ORC_T_LM: p = m->lm; n = V * d; break;
    case ORC_T_GF: p = m->gf; n = d; break;
    default:
      if (!L) break;
      switch (tensor_id) {
        case ORC_T_G1: p = L->g1; n = d; break;
        case ORC_T_WQ: p = L->wq; n = nq * d; break;
        case ORC_T_WK: p = L->wk; n = nkv * d; break;
        case ORC_T_WV: p = L->wv; n = nkv * d; break;
        case ORC_T_GQ: p = L->gq; n = hd; break;
        case ORC_T_GK: p = L->gk; n = hd; break;
        case ORC_T_WO: p = L->wo; n = d * nq; break;
        case ORC_T_G2: p = L->g2; n = d; break;
        case ORC_T_WG: p = L->wg; n = F * d; break;
        case ORC_T_WU: p = L->wu; n = F * d; break;
        case ORC_T_WD: p = L->wd; n = d * F; break;
        default: break;
      }
  }
  if (n_elems) *n_elems = n;
  return p;
}

/* ------------------------------------------------------- sequence state */

orc_seq *orc_seq_new(const orc_model *m, int max_hist) {
  orc_seq *s = (orc_seq *)calloc(1, sizeof(orc_seq));
  if (!s) return NULL;
  const orc_cfg *c = &m->cfg;
  size_t n = (size_t)c->n_layers * c->n_kv_heads * c->max_ctx * c->head_dim;
  s->model = m;
  s->max_hist = max_hist;
  s->hist = (int32_t *)calloc(max_hist > 0 ? max_hist : 1, sizeof(int32_t));
  s->kc = (double *)calloc(n ? n : 1, sizeof(double));
  s->vc = (double *)calloc(n ? n : 1, sizeof(double));
  return s;
}

void orc_seq_free(orc_seq *s) {
  if (!s) return;
  free(s->hist); free(s->kc); free(s->vc); free(s);
}

int32_t orc_seq_kv_len(const orc_seq *s) { return s->kv_len; }
int32_t orc_seq_hist_len(const orc_seq *s) { return s->hist_len; }
int32_t *orc_seq_hist(orc_seq *s) { return s->hist; }
double *orc_seq_kcache(orc_seq *s) { return s->kc; }
double *orc_seq_vcache(orc_seq *s) { return s->vc; }

void orc_seq_reset(orc_seq *s) { s->kv_len = 0; s->hist_len = 0; }

/* Rollback (Alg. 1 "rollback M_q", Alg. 2 "rollback both models"): forget the KV rows
 * and the history tokens beyond the given lengths; -1 leaves a length as it is. */
int orc_seq_truncate(orc_seq *s, int kv_len, int hist_len) {
  if (kv_len > s->kv_len || hist_len > s->hist_len) return -1;
  if (kv_len >= 0) s->kv_len = kv_len;
  if (hist_len >= 0) s->hist_len = hist_len;
  return 0;
}

int orc_seq_hist_set(orc_seq *s, const int32_t *tok, int n) {
  if (n < 0 || n > s->max_hist) return -1;
  memcpy(s->hist, tok, sizeof(int32_t) * (size_t)n);
  s->hist_len = n;
  return 0;
}

static size_t kv_index(const orc_cfg *c, int layer, int kvh, int slot) {
  return (((size_t)layer * c->n_kv_heads + kvh) * c->max_ctx + slot) * c->head_dim;
}

/* ------------------------------------------------------------ layer pieces */

/* rmsnorm(x)_i = x_i * g_i / sqrt(mean(x^2) + eps) */
void orc_rmsnorm(const double *x, const float *g, int n, double eps, double *out) {
  double ss = 0.0;
  for (int i = 0; i < n; ++i) ss += x[i] * x[i];
  double r = 1.0 / sqrt(ss / n + eps);
  for (int i = 0; i < n; ++i) out[i] = x[i] * r * (double)g[i];
}

/* Rotary embedding, half-split pairing: dims (i, i + hd/2) rotate by the angle
 * pos * base^(-2i/hd).  cos/sin are taken from fp32-rounded table entries (the
 * table a device would hold). */
void orc_rope(double *v, int hd, int pos, double base) {
  int half = hd / 2;
  for (int i = 0; i < half; ++i) {
    double theta = pow(base, -2.0 * i / hd);
    double ang = (double)pos * theta;
    double c = (double)(float)cos(ang), s = (double)(float)sin(ang);
    double a = v[i], b = v[i + half];
    v[i] = a * c - b * s;
    v[i + half] = a * s + b * c;
  }
}

/* y[n] = sum_k W[n][k] x[k], k ascending, fp64 accumulate */
static void matvec(const float *W, const double *x, int N, int K, double *y) {
#pragma omp parallel for schedule(static)
  for (int n = 0; n < N; ++n) {
    const float *w = W + (size_t)n * K;
    double acc = 0.0;
    for (int k = 0; k < K; ++k) acc += (double)w[k] * x[k];
    y[n] = acc;
  }
}

/* ---------------------------------------------------------------- forward */

/* One window row through one layer.  h is the fp64 residual stream of this row,
 * pos = its absolute position = the KV slot it writes. */
static void layer_row(const orc_model *m, orc_seq *s, int l, int pos, double *h, double *scr) {
  const orc_cfg *c = &m->cfg;
  const orc_layer *L = &m->layers[l];
  const int d = c->d_model, hd = c->head_dim, H = c->n_q_heads, Hkv = c->n_kv_heads;
  const int F = c->d_ffn, g = H / Hkv;
  double *a = scr;             /* d     */
  double *q = a + d;           /* H*hd  */
  double *kk = q + H * hd;     /* Hkv*hd */
  double *vv = kk + Hkv * hd;  /* Hkv*hd */
  double *att = vv + Hkv * hd; /* H*hd  */
  double *o = att + H * hd;    /* d     */
  double *gt = o + d;          /* F     */
  double *up = gt + F;         /* F     */
  double *sc = up + F;         /* max_ctx */

  orc_rmsnorm(h, L->g1, d, c->rms_eps, a);
  for (int i = 0; i < d; ++i) a[i] = rnd(c, a[i]); /* r1 */
  matvec(L->wq, a, H * hd, d, q);
  matvec(L->wk, a, Hkv * hd, d, kk);
  matvec(L->wv, a, Hkv * hd, d, vv);
  if (c->qk_norm) {
    for (int hh = 0; hh < H; ++hh) orc_rmsnorm(q + hh * hd, L->gq, hd, c->rms_eps, q + hh * hd);
    for (int hh = 0; hh < Hkv; ++hh) orc_rmsnorm(kk + hh * hd, L->gk, hd, c->rms_eps, kk + hh * hd);
  }
  for (int hh = 0; hh < H; ++hh) orc_rope(q + hh * hd, hd, pos, c->rope_base);
  for (int hh = 0; hh < Hkv; ++hh) orc_rope(kk + hh * hd, hd, pos, c->rope_base);
  for (int i = 0; i < H * hd; ++i) q[i] = rnd(c, q[i]); /* r2 */
  for (int hh = 0; hh < Hkv; ++hh) {
    double *kd = s->kc + kv_index(c, l, hh, pos), *vd = s->vc + kv_index(c, l, hh, pos);
    for (int i = 0; i < hd; ++i) {
      kd[i] = rnd(c, kk[hh * hd + i]); /* r2 */
      vd[i] = rnd(c, vv[hh * hd + i]); /* r2 */
    }
  }
  /* attention of this row over slots 0..pos (its own slot included) */
  const double scale = 1.0 / sqrt((double)hd);
  for (int hh = 0; hh < H; ++hh) {
    const int kvh = hh / g;
    const double *qh = q + hh * hd;
    double mx = -INFINITY;
    for (int t = 0; t <= pos; ++t) {
      const double *kt = s->kc + kv_index(c, l, kvh, t);
      double dot = 0.0;
      for (int i = 0; i < hd; ++i) dot += qh[i] * kt[i];
      sc[t] = dot * scale;
      if (sc[t] > mx) mx = sc[t];
    }
    double den = 0.0;
    for (int t = 0; t <= pos; ++t) { sc[t] = exp(sc[t] - mx); den += sc[t]; }
    for (int t = 0; t <= pos; ++t) sc[t] = sc[t] / den;
    for (int i = 0; i < hd; ++i) {
      double acc = 0.0;
      for (int t = 0; t <= pos; ++t) acc += sc[t] * s->vc[kv_index(c, l, kvh, t) + i];
      att[hh * hd + i] = rnd(c, acc); /* r3 */
    }
  }
  matvec(L->wo, att, d, H * hd, o);
  for (int i = 0; i < d; ++i) h[i] += o[i];

  orc_rmsnorm(h, L->g2, d, c->rms_eps, a);
  for (int i = 0; i < d; ++i) a[i] = rnd(c, a[i]); /* r1 */
  matvec(L->wg, a, F, d, gt);
  matvec(L->wu, a, F, d, up);
  for (int i = 0; i < F; ++i) {
    double silu = gt[i] / (1.0 + exp(-gt[i]));
    gt[i] = rnd(c, silu * up[i]); /* r4 */
  }
  matvec(L->wd, gt, d, F, o);
  for (int i = 0; i < d; ++i) h[i] += o[i];
}

/* Verify forward: window[0] is the pending token (last emitted, KV not yet
 * written), window[1..k) the drafted tokens.  Row j sits at position
 * kv_len + j, writes KV slot kv_len + j, and attends to slots 0..kv_len+j.
 * logits[j][:] is the target's prediction for the token after window[j].
 * kv_len is NOT advanced (commit does that); rows are processed layer by
 * layer, each row with the same arithmetic and loop order as a 1-row call.
 * hidden_opt (may be NULL) receives the final-norm input rows [k][d]. */
int orc_verify_block(const orc_model *m, orc_seq *s, const int32_t *window, int k,
                     double *logits, double *hidden_opt) {
  const orc_cfg *c = &m->cfg;
  const int d = c->d_model, V = c->vocab;
  if (k < 1 || s->kv_len + k > c->max_ctx) return -1;
  for (int j = 0; j < k; ++j)
    if (window[j] < 0 || window[j] >= V) return -2;
  size_t nscr = (size_t)3 * d + 2 * (size_t)c->n_q_heads * c->head_dim +
                2 * (size_t)c->n_kv_heads * c->head_dim + 2 * (size_t)c->d_ffn + c->max_ctx;
  double *scr = (double *)malloc(sizeof(double) * nscr);
  double *h = (double *)malloc(sizeof(double) * (size_t)k * d);
  if (!scr || !h) { free(scr); free(h); return -3; }
  for (int j = 0; j < k; ++j)
    for (int i = 0; i < d; ++i) h[(size_t)j * d + i] = (double)m->emb[(size_t)window[j] * d + i];
  for (int l = 0; l < c->n_layers; ++l)
    for (int j = 0; j < k; ++j) layer_row(m, s, l, s->kv_len + j, h + (size_t)j * d, scr);
  for (int j = 0; j < k; ++j) {
    double *a = scr;
    if (hidden_opt) memcpy(hidden_opt + (size_t)j * d, h + (size_t)j * d, sizeof(double) * d);
    orc_rmsnorm(h + (size_t)j * d, m->gf, d, c->rms_eps, a);
    for (int i = 0; i < d; ++i) a[i] = rnd(c, a[i]); /* r1 */
    matvec(m->lm, a, V, d, logits + (size_t)j * V);
  }
  free(scr); free(h);
  return 0;
}

/* ----------------------------------------------------------------- accept */

/* argmax with lowest id on exact ties; also the gap to the runner-up */
static int argmax_gap(const double *z, int V, double *gap) {
  int best = 0; double b1 = z[0], b2 = -INFINITY;
  for (int v = 1; v < V; ++v) {
    if (z[v] > b1) { b2 = b1; b1 = z[v]; best = v; }
    else if (z[v] > b2) b2 = z[v];
  }
  if (gap) *gap = b1 - b2;
  return best;
}

/* Greedy acceptance.  y_j = argmax(logits[j]); n_acc = number of leading
 * drafts with window[j+1] == y_j; emit = accepted drafts then y_{n_acc};
 * guide = y_0..y_{k-1}; margin[j] = top-2 logit gap of row j. */
void orc_accept_greedy(const double *logits, int k, int V, const int32_t *window,
                       int32_t *n_acc, int32_t *emit, int32_t *guide, double *margin) {
  for (int j = 0; j < k; ++j) guide[j] = argmax_gap(logits + (size_t)j * V, V, margin ? margin + j : NULL);
  int n = 0;
  while (n < k - 1 && window[n + 1] == guide[n]) ++n;
  for (int i = 0; i < n; ++i) emit[i] = window[i + 1];
  emit[n] = guide[n];
  for (int i = n + 1; i < k; ++i) emit[i] = -1;
  *n_acc = n;
}

static void softmax_T(const double *z, int V, double T, double *p) {
  double mx = -INFINITY, den = 0.0;
  for (int v = 0; v < V; ++v) if (z[v] / T > mx) mx = z[v] / T;
  for (int v = 0; v < V; ++v) { p[v] = exp(z[v] / T - mx); den += p[v]; }
  for (int v = 0; v < V; ++v) p[v] /= den;
}

/* Standard Gumbel noise for vocab entry v of row j: Philox counter
 * (step, b, j, 1 + v/4), word v%4. */
static double gumbel(uint64_t seed, uint64_t step, int b, int j, int v) {
  uint32_t ctr[4] = {(uint32_t)step, (uint32_t)b, (uint32_t)j, (uint32_t)(1 + v / 4)};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t o[4];
  orc_philox4x32_10(ctr, key, o);
  return -log(-log(u01(o[v & 3])));
}

/* Draw from weights w (not normalised) as argmax_v [log w_v + Gumbel_v] over
 * w_v > 0 -- an exact categorical sample (Gumbel-max).  Returns -1 when every
 * weight is zero.  gap = winner's score minus the runner-up's. */
static int gumbel_draw(const double *w, int V, uint64_t seed, uint64_t step, int b, int j, double *gap) {
  int best = -1; double b1 = -INFINITY, b2 = -INFINITY;
  for (int v = 0; v < V; ++v) {
    if (!(w[v] > 0.0)) continue;
    double sc = log(w[v]) + gumbel(seed, step, b, j, v);
    if (sc > b1) { b2 = b1; b1 = sc; best = v; }
    else if (sc > b2) b2 = sc;
  }
  if (gap) *gap = b1 - b2;
  return best;
}

/* Speculative-sampling acceptance at temperature T.
 * p_j = softmax(logits[j]/T).  q (may be NULL) holds the draft distributions
 * [k-1][V]; NULL means the drafts were proposed deterministically (retrieved),
 * i.e. q_j is one-hot at the draft.  For j = 0..k-2 with x = window[j+1]:
 * accept iff u_j * q_j(x) < p_j(x), u_j = Philox(step, b, j, 0) word 0.
 * At the first rejected row n the output token is drawn from max(0, p_n - q_n)
 * (from p_n if that is identically zero); with no rejection n = k-1 and the
 * extra token is drawn from p_{k-1}.  Nothing of the rows after n is used:
 * guide[j] for j <= n is a draw from p_j made with row j's Gumbel noise (the
 * target's own sample at that row), and -1 for j > n.
 * Diagnostics for parity tests (none of them feeds a decision):
 * acc_margin[j] = |u_j q_j(x) - p_j(x)| for the rows tested (else -1);
 * draw_gap = Gumbel-max score gap of the emitted token's draw;
 * guide_gap (may be NULL) [k]: the same gap for row j's own draw guide[j], -1 for j > n. */
void orc_accept_sample(const double *logits, int k, int V, const int32_t *window,
                       const float *q, double T, uint64_t seed, uint64_t step, int b,
                       int32_t *n_acc, int32_t *emit, int32_t *guide,
                       double *acc_margin, double *draw_gap, double *guide_gap) {
  double *p = (double *)malloc(sizeof(double) * V);
  double *w = (double *)malloc(sizeof(double) * V);
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  int n = k - 1;
  for (int j = 0; j < k; ++j) {
    guide[j] = -1; emit[j] = -1;
    if (acc_margin) acc_margin[j] = -1.0;
    if (guide_gap) guide_gap[j] = -1.0;
  }
  for (int j = 0; j < k - 1; ++j) {
    const int x = window[j + 1];
    softmax_T(logits + (size_t)j * V, V, T, p);
    uint32_t ctr[4] = {(uint32_t)step, (uint32_t)b, (uint32_t)j, 0u}, o[4];
    orc_philox4x32_10(ctr, key, o);
    double u = u01(o[0]);
    double qx = q ? (double)q[(size_t)j * V + x] : 1.0;
    if (acc_margin) acc_margin[j] = fabs(u * qx - p[x]);
    if (!(u * qx < p[x])) { n = j; break; }
  }
  for (int j = 0; j <= n; ++j) {
    softmax_T(logits + (size_t)j * V, V, T, p);
    guide[j] = gumbel_draw(p, V, seed, step, b, j, guide_gap ? guide_gap + j : NULL);
  }
  softmax_T(logits + (size_t)n * V, V, T, p);
  int tok;
  if (n < k - 1) { /* rejected at row n: residual */
    const int x = window[n + 1];
    for (int v = 0; v < V; ++v) {
      double qv = q ? (double)q[(size_t)n * V + v] : (v == x ? 1.0 : 0.0);
      w[v] = p[v] - qv > 0.0 ? p[v] - qv : 0.0;
    }
    tok = gumbel_draw(w, V, seed, step, b, n, draw_gap);
    if (tok < 0) tok = gumbel_draw(p, V, seed, step, b, n, draw_gap);
  } else {
    tok = gumbel_draw(p, V, seed, step, b, n, draw_gap);
  }
  for (int i = 0; i < n; ++i) emit[i] = window[i + 1];
  emit[n] = tok;
  *n_acc = n;
  free(p); free(w);
}

/* --------------------------------------------------------------- retrieve */

/* Longest-suffix n-gram search of the history in itself.  For n from
 * min(n_max, len-1) down to n_min: every start s in [0, len-n-1] with
 * hist[s..s+n) == hist[len-n..len) is a candidate (the suffix itself is not,
 * so each candidate has at least one following token); its continuation is
 * the next min(max_cont, len-s-n) tokens.  The first n with a candidate wins;
 * among its candidates the longest continuation wins, then the latest start.
 * Miss: cont_len = 0, match_n = 0, match_pos = -1. */
void orc_retrieve(const int32_t *hist, int len, int n_max, int n_min, int max_cont,
                  int32_t *cont, int32_t *cont_len, int32_t *match_n, int32_t *match_pos) {
  *cont_len = 0; *match_n = 0; *match_pos = -1;
  if (n_min < 1) n_min = 1;
  int n0 = n_max < len - 1 ? n_max : len - 1;
  for (int n = n0; n >= n_min; --n) {
    int best_s = -1, best_c = 0;
    for (int s = 0; s + n <= len - 1; ++s) {
      int eq = 1;
      for (int i = 0; i < n; ++i)
        if (hist[s + i] != hist[len - n + i]) { eq = 0; break; }
      if (!eq) continue;
      int c = len - s - n; if (c > max_cont) c = max_cont;
      if (c > best_c || (c == best_c && s > best_s)) { best_c = c; best_s = s; }
    }
    if (best_s >= 0) {
      for (int i = 0; i < best_c; ++i) cont[i] = hist[best_s + n + i];
      *cont_len = best_c; *match_n = n; *match_pos = best_s;
      return;
    }
  }
}

/* ----------------------------------------------------------------- commit */

/* ------------------------------------------------- hierarchical datastore
 *
 * Alg. 3 (Retrieval Cache Mechanism) and Sec. 4.3.  Three token tiers are searched in a
 * fixed priority for every n-gram length, longest first; only if no length hits in any
 * tier does the search fall back to the plain search of the sequence in itself:
 *   tier 0  C_prefix    a static token stream (the prior), shared by all sequences
 *   tier 1  C_dynamic   the tokens generated in this session: hist[prompt_len .. len)
 *   tier 2  C_rejected  the session's rejected draft chains
 *   tier 3  fallback    the whole sequence (prompt + generated): orc_retrieve
 * A tier is a token buffer; -1 separates segments (documents, rejected chains): an n-gram
 * never contains a separator and a continuation stops in front of one.  Inside a tier the
 * occurrence with the longest continuation (<= max_cont) wins, then the latest one -- the
 * same rule as orc_retrieve.  The key is always the last n tokens of hist. */

/* best occurrence of key[0..n) in buf[0..len) whose n-gram starts at or after lo and ends
 * before hi_end (the key's own position must be excluded by the caller through hi_end) */
static int tier_best(const int32_t *buf, int len, int lo, int hi_end, const int32_t *key, int n, int max_cont,
                     int *best_c) {
  int best_s = -1; *best_c = 0;
  for (int s = lo; s + n <= hi_end; ++s) {
    int eq = 1;
    for (int i = 0; i < n; ++i) if (buf[s + i] != key[i]) { eq = 0; break; }
    if (!eq) continue;
    int c = 0;
    while (c < max_cont && s + n + c < len && buf[s + n + c] >= 0) ++c;
    if (c < 1) continue;
    if (c > *best_c || (c == *best_c && s > best_s)) { *best_c = c; best_s = s; }
  }
  return best_s;
}

void orc_retrieve_tiered(const int32_t *prior, int prior_len, const int32_t *hist, int len, int prompt_len,
                         const int32_t *rej, int rej_len, int n_max, int n_min, int max_cont,
                         int32_t *cont, int32_t *cont_len, int32_t *match_n, int32_t *match_pos,
                         int32_t *match_tier) {
  *cont_len = 0; *match_n = 0; *match_pos = -1; *match_tier = -1;
  if (n_min < 1) n_min = 1;
  if (len < 1) return;
  int n0 = n_max < len ? n_max : len;
  for (int n = n0; n >= n_min; --n) {
    const int32_t *key = hist + len - n;
    for (int tier = 0; tier < 3; ++tier) {
      const int32_t *buf; int blen, lo, hi_end;
      if (tier == 0) { buf = prior; blen = prior_len; lo = 0; hi_end = prior_len; }
      else if (tier == 1) { buf = hist; blen = len; lo = prompt_len; hi_end = len - 1; }   /* not the key itself */
      else { buf = rej; blen = rej_len; lo = 0; hi_end = rej_len; }
      if (!buf || blen <= 0) continue;
      int c, s = tier_best(buf, blen, lo, hi_end, key, n, max_cont, &c);
      if (s >= 0) {
        for (int i = 0; i < c; ++i) cont[i] = buf[s + n + i];
        *cont_len = c; *match_n = n; *match_pos = s; *match_tier = tier;
        return;
      }
    }
  }
  orc_retrieve(hist, len, n_max, n_min, max_cont, cont, cont_len, match_n, match_pos);
  if (*match_n > 0) *match_tier = 3;
}

/* Cache update of Alg. 3 for the rejected tier: after a window (pending token + drafts) was
 * verified with n_acc drafts accepted, the drafts behind the first rejection,
 * window[n_acc+1 .. n_draft], are appended as one segment: up to ctx_tokens tokens of the text
 * in front of them (history followed by the accepted drafts), the rejected tokens, a
 * separator.  Nothing is stored when no draft was rejected or the segment does not fit.
 * hist is the history BEFORE the commit (it ends with the pending token = window[0]).
 * Returns the new length of the tier. */
int orc_rejected_append(int32_t *rej, int rej_len, int rej_cap, const int32_t *hist, int len,
                        const int32_t *window, int n_acc, int n_draft, int ctx_tokens) {
  int n_rej = n_draft - n_acc;
  if (n_rej < 1) return rej_len;
  /* text in front of the rejected tokens: hist[0..len) + window[1..n_acc] */
  int avail = len + n_acc;
  int nctx = ctx_tokens < avail ? ctx_tokens : avail;
  if (rej_len + nctx + n_rej + 1 > rej_cap) return rej_len;
  for (int i = 0; i < nctx; ++i) {
    int p = avail - nctx + i;               /* position in hist + accepted */
    rej[rej_len++] = p < len ? hist[p] : window[1 + (p - len)];
  }
  for (int i = 0; i < n_rej; ++i) rej[rej_len++] = window[n_acc + 1 + i];
  rej[rej_len++] = -1;
  return rej_len;
}

/* Keep the first n_keep window rows' KV (the pending token and the accepted
 * drafts), drop the rest (they are simply overwritten by the next window), and
 * append the n_emit emitted tokens to the history. */
int orc_commit(orc_seq *s, int n_keep, const int32_t *emit, int n_emit) {
  if (n_keep < 0 || s->kv_len + n_keep > s->model->cfg.max_ctx) return -1;
  if (n_emit < 0 || s->hist_len + n_emit > s->max_hist) return -2;
  s->kv_len += n_keep;
  for (int i = 0; i < n_emit; ++i) s->hist[s->hist_len + i] = emit[i];
  s->hist_len += n_emit;
  return 0;
}
