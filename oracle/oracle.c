/*
 * oracle.c -- plain CPU oracle of a LLaMA-architecture decoder at batch 1.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct
 * statement of what the GPU hot path must compute.  It shares no code with
 * the HIP library and must never be called from the product path; only the
 * tests, the smoke check and the benchmark's CPU-baseline leg use it.
 *
 * The paper names the model (LLaMA-2 7B, Sec. IV-E "Benchmark Configuration")
 * and the operator classes of one decoding step (Sec. III-A: linear
 * projections, normalisation, matrix multiplications, attention scores;
 * KV-cache update, positional-embedding extension, token sampling; Alg. 1:
 * one token per step, t_i = f_decode(h_i)).  It prints no equations, so each
 * operator below is the standard definition of that operator for the LLaMA
 * architecture, written as the plainest loop that states it:
 *
 *   RMSNorm   a_i = x_i * (1/sqrt(mean_j x_j^2 + eps)) * g_i
 *   linear    y = W x,  W row-major [out, in]
 *   RoPE      pairs (j, j + d_h/2) of every head rotated by pos * theta^(-2j/d_h)
 *   attention s_u = q.K_u / sqrt(d_h), u = 0..pos; softmax with max
 *             subtraction; o = sum_u w_u V_u
 *   SwiGLU    m_i = silu(g_i) * u_i,  silu(z) = z / (1 + exp(-z))
 *   sampling  greedy: smallest index among the maxima of the logits
 *
 * One source, two builds: `real` is float by default (the fp32 oracle the GPU
 * path is judged against) and double with -DORACLE_F64 (used by the CPU tests
 * to bound the fp32 build's own rounding error).  There is no blocking, no
 * fusion and no reordering; OpenMP only spreads independent output rows /
 * heads over threads.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef ORACLE_F64
typedef double real;
#define R_EXP exp
#define R_SQRT sqrt
#else
typedef float real;
#define R_EXP expf
#define R_SQRT sqrtf
#endif

enum { ORACLE_DT_F32 = 0, ORACLE_DT_F16 = 1 };

typedef struct {
  int32_t n_layers, d_model, n_heads, head_dim, ffn_hidden, vocab, max_seq;
  float rope_theta, rms_eps;
} oracle_config;

typedef struct {
  const void *attn_norm, *wq, *wk, *wv, *wo, *ffn_norm, *w_gate, *w_up, *w_down;
} oracle_layer;

typedef struct {
  const void *tok_emb;
  const oracle_layer *layers;
  const void *final_norm;
  const void *lm_head;
  int32_t dtype; /* ORACLE_DT_*: element type of every weight array */
} oracle_weights;

typedef struct {
  oracle_config cfg;
  oracle_weights w;
  oracle_layer *layers; /* owned copy of the per-layer pointer table */
  real *kcache, *vcache; /* [layer][pos][d_model] */
  int32_t pos;          /* number of positions already in the cache */
  real *x, *a, *q, *k, *v, *o, *t, *g, *u, *m, *scores;
} oracle_model;

int oracle_real_bytes(void) { return (int)sizeof(real); }

/* IEEE-754 binary16 bit pattern -> value, by the format's definition:
 * sign, 5-bit exponent (bias 15), 10-bit fraction; exponent 0 is subnormal
 * (fraction * 2^-24), exponent 31 is inf / NaN. */
float oracle_half_to_float(uint16_t h) {
  int sign = (h >> 15) & 1;
  int e = (h >> 10) & 0x1f;
  int f = h & 0x3ff;
  double val;
  if (e == 0)
    val = ldexp((double)f, -24);
  else if (e == 31)
    val = f ? (double)NAN : (double)INFINITY;
  else
    val = ldexp((double)(f + 1024), e - 25);
  return (float)(sign ? -val : val);
}

/* All 65536 binary16 values, filled once from the definition above so that a
 * 7B-sized matvec does not pay for ldexp per element. */
static float h2f_table[65536];
static int h2f_ready = 0;
static void h2f_init(void) {
  if (h2f_ready) return;
#pragma omp critical(oracle_h2f)
  {
    if (!h2f_ready) {
      for (uint32_t b = 0; b < 65536u; ++b) h2f_table[b] = oracle_half_to_float((uint16_t)b);
      h2f_ready = 1;
    }
  }
}

static inline real wread(const void *base, size_t i, int dtype) {
  if (dtype == ORACLE_DT_F16) return (real)h2f_table[((const uint16_t *)base)[i]];
  return (real)((const float *)base)[i];
}

/* a_i = x_i * (1/sqrt(mean(x^2) + eps)) * g_i */
void oracle_rmsnorm(const real *x, const void *g, int dtype, int n, float eps, real *out) {
  h2f_init();
  real ss = 0;
  for (int j = 0; j < n; ++j) ss += x[j] * x[j];
  real r = ss / (real)n;
  real inv = (real)1 / R_SQRT(r + (real)eps);
  for (int i = 0; i < n; ++i) out[i] = x[i] * inv * wread(g, (size_t)i, dtype);
}

/* y = W x, W row-major [n_out, n_in] */
void oracle_matvec(const void *W, int dtype, int n_out, int n_in, const real *x, real *y) {
  h2f_init();
#pragma omp parallel for schedule(static)
  for (int i = 0; i < n_out; ++i) {
    real acc = 0;
    size_t row = (size_t)i * (size_t)n_in;
    for (int j = 0; j < n_in; ++j) acc += wread(W, row + (size_t)j, dtype) * x[j];
    y[i] = acc;
  }
}

/* Rotary position embedding, "rotate-half" pairing: within every head the
 * pair (j, j + d_h/2) is rotated by the angle pos * theta^(-2j/d_h).  The
 * angle and its cosine/sine are taken in double and rounded to `real`. */
void oracle_rope(real *vec, int n_heads, int head_dim, int pos, float theta) {
  int half = head_dim / 2;
  for (int h = 0; h < n_heads; ++h) {
    real *p = vec + (size_t)h * head_dim;
    for (int j = 0; j < half; ++j) {
      double phi = (double)pos * pow((double)theta, -2.0 * (double)j / (double)head_dim);
      real c = (real)cos(phi), s = (real)sin(phi);
      real lo = p[j], hi = p[j + half];
      p[j] = lo * c - hi * s;
      p[j + half] = hi * c + lo * s;
    }
  }
}

/* One head of causal attention over n_keys cached rows.  K and V rows of this
 * head are `stride` reals apart.  w_out (nullable) receives the softmax row. */
void oracle_attention_head(const real *q, const real *K, const real *V, int n_keys, int head_dim,
                           int stride, real *o, real *w_out) {
  real *s = (real *)malloc(sizeof(real) * (size_t)n_keys);
  real scale = (real)1 / R_SQRT((real)head_dim);
  real mx = -INFINITY;
  for (int u = 0; u < n_keys; ++u) {
    real dot = 0;
    for (int c = 0; c < head_dim; ++c) dot += q[c] * K[(size_t)u * stride + c];
    s[u] = dot * scale;
    if (s[u] > mx) mx = s[u];
  }
  real den = 0;
  for (int u = 0; u < n_keys; ++u) {
    s[u] = R_EXP(s[u] - mx);
    den += s[u];
  }
  for (int u = 0; u < n_keys; ++u) s[u] = s[u] / den;
  for (int c = 0; c < head_dim; ++c) {
    real acc = 0;
    for (int u = 0; u < n_keys; ++u) acc += s[u] * V[(size_t)u * stride + c];
    o[c] = acc;
  }
  if (w_out) memcpy(w_out, s, sizeof(real) * (size_t)n_keys);
  free(s);
}

/* m_i = silu(g_i) * u_i */
void oracle_swiglu(const real *g, const real *u, int n, real *m) {
  for (int i = 0; i < n; ++i) m[i] = g[i] / ((real)1 + R_EXP(-g[i])) * u[i];
}

/* Greedy choice: smallest index among the maxima. */
int oracle_argmax(const real *v, int n) {
  int best = 0;
  for (int i = 1; i < n; ++i)
    if (v[i] > v[best]) best = i;
  return best;
}

void oracle_model_free(oracle_model *m) {
  if (!m) return;
  free(m->layers);
  free(m->kcache);
  free(m->vcache);
  free(m->x); free(m->a); free(m->q); free(m->k); free(m->v); free(m->o); free(m->t);
  free(m->g); free(m->u); free(m->m); free(m->scores);
  free(m);
}

/* The weights stay where the caller put them (no copy); the caller keeps them
 * alive while the model exists. */
oracle_model *oracle_model_new(const oracle_config *cfg, const oracle_weights *w) {
  if (!cfg || !w) return NULL;
  if (cfg->n_layers < 1 || cfg->d_model < 1 || cfg->n_heads < 1 || cfg->head_dim < 2 ||
      (cfg->head_dim & 1) || cfg->n_heads * cfg->head_dim != cfg->d_model || cfg->ffn_hidden < 1 ||
      cfg->vocab < 1 || cfg->max_seq < 1)
    return NULL;
  oracle_model *m = (oracle_model *)calloc(1, sizeof(oracle_model));
  if (!m) return NULL;
  m->cfg = *cfg;
  m->w = *w;
  m->layers = (oracle_layer *)malloc(sizeof(oracle_layer) * (size_t)cfg->n_layers);
  memcpy(m->layers, w->layers, sizeof(oracle_layer) * (size_t)cfg->n_layers);
  m->w.layers = m->layers;
  size_t d = (size_t)cfg->d_model, f = (size_t)cfg->ffn_hidden;
  size_t kv = (size_t)cfg->n_layers * (size_t)cfg->max_seq * d;
  m->kcache = (real *)calloc(kv, sizeof(real));
  m->vcache = (real *)calloc(kv, sizeof(real));
  m->x = (real *)calloc(d, sizeof(real));
  m->a = (real *)calloc(d, sizeof(real));
  m->q = (real *)calloc(d, sizeof(real));
  m->k = (real *)calloc(d, sizeof(real));
  m->v = (real *)calloc(d, sizeof(real));
  m->o = (real *)calloc(d, sizeof(real));
  m->t = (real *)calloc(d, sizeof(real));
  m->g = (real *)calloc(f, sizeof(real));
  m->u = (real *)calloc(f, sizeof(real));
  m->m = (real *)calloc(f, sizeof(real));
  m->scores = NULL;
  if (!m->kcache || !m->vcache || !m->x || !m->a || !m->q || !m->k || !m->v || !m->o || !m->t ||
      !m->g || !m->u || !m->m) {
    oracle_model_free(m);
    return NULL;
  }
  return m;
}

void oracle_model_reset(oracle_model *m) { m->pos = 0; }
int oracle_model_pos(const oracle_model *m) { return m->pos; }
/* which: 0 = keys, 1 = values; rows [pos][d_model] of one layer */
const real *oracle_model_kv(const oracle_model *m, int layer, int which) {
  size_t off = (size_t)layer * (size_t)m->cfg.max_seq * (size_t)m->cfg.d_model;
  return (which ? m->vcache : m->kcache) + off;
}

/*
 * One decoding step: feed `token` at position p = (number of cached
 * positions), append its keys/values to the cache, return the greedy next
 * token.  logits_out [vocab] and hidden_out [d_model] (the residual stream
 * before the final norm) are optional.  Returns -1 on a bad token or a full
 * cache.
 */
int oracle_model_step(oracle_model *m, int token, real *logits_out, real *hidden_out) {
  const oracle_config *c = &m->cfg;
  int d = c->d_model, H = c->n_heads, dh = c->head_dim, F = c->ffn_hidden, V = c->vocab;
  int dt = m->w.dtype;
  int p = m->pos;
  h2f_init();
  if (token < 0 || token >= V || p >= c->max_seq) return -1;

  for (int i = 0; i < d; ++i) m->x[i] = wread(m->w.tok_emb, (size_t)token * d + i, dt);

  for (int l = 0; l < c->n_layers; ++l) {
    const oracle_layer *L = &m->layers[l];
    real *Kc = m->kcache + (size_t)l * c->max_seq * d;
    real *Vc = m->vcache + (size_t)l * c->max_seq * d;

    oracle_rmsnorm(m->x, L->attn_norm, dt, d, c->rms_eps, m->a);
    oracle_matvec(L->wq, dt, d, d, m->a, m->q);
    oracle_matvec(L->wk, dt, d, d, m->a, m->k);
    oracle_matvec(L->wv, dt, d, d, m->a, m->v);
    oracle_rope(m->q, H, dh, p, c->rope_theta);
    oracle_rope(m->k, H, dh, p, c->rope_theta);
    memcpy(Kc + (size_t)p * d, m->k, sizeof(real) * (size_t)d);
    memcpy(Vc + (size_t)p * d, m->v, sizeof(real) * (size_t)d);

#pragma omp parallel for schedule(static)
    for (int h = 0; h < H; ++h)
      oracle_attention_head(m->q + (size_t)h * dh, Kc + (size_t)h * dh, Vc + (size_t)h * dh, p + 1,
                            dh, d, m->o + (size_t)h * dh, NULL);

    oracle_matvec(L->wo, dt, d, d, m->o, m->t);
    for (int i = 0; i < d; ++i) m->x[i] += m->t[i];

    oracle_rmsnorm(m->x, L->ffn_norm, dt, d, c->rms_eps, m->a);
    oracle_matvec(L->w_gate, dt, F, d, m->a, m->g);
    oracle_matvec(L->w_up, dt, F, d, m->a, m->u);
    oracle_swiglu(m->g, m->u, F, m->m);
    oracle_matvec(L->w_down, dt, d, F, m->m, m->t);
    for (int i = 0; i < d; ++i) m->x[i] += m->t[i];
  }

  if (hidden_out) memcpy(hidden_out, m->x, sizeof(real) * (size_t)d);
  oracle_rmsnorm(m->x, m->w.final_norm, dt, d, c->rms_eps, m->a);
  real *logits = logits_out ? logits_out : (real *)malloc(sizeof(real) * (size_t)V);
  oracle_matvec(m->w.lm_head, dt, V, d, m->a, logits);
  int tok = oracle_argmax(logits, V);
  if (!logits_out) free(logits);
  m->pos = p + 1;
  return tok;
}
