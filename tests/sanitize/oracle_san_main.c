/*
 * Drives every entry point of the CPU oracle (oracle/oracle.c, compiled into this translation unit)
 * under AddressSanitizer + UndefinedBehaviorSanitizer on the host: exact-size heap buffers, so any
 * read or write past an operand, the KV cache or the logits aborts the run.  Host only; no GPU.
 *
 *   gcc -O1 -g -fsanitize=address,undefined -fno-sanitize-recover=all -fopenmp \
 *       [-DORACLE_F64] tests/sanitize/oracle_san_main.c -lm -o oracle_san && ./oracle_san
 */
#include "../../oracle/oracle.c"

#include <stdio.h>

static uint32_t rng_state = 12345u;
static float rnd(void) {   /* uniform in [-1, 1): only bounds matter here, not the distribution */
  rng_state = rng_state * 1664525u + 1013904223u;
  return (float)(rng_state >> 8) / 8388608.0f - 1.0f;
}
static float *fvec(size_t n, float scale) {
  float *p = (float *)malloc(n * sizeof(float));
  for (size_t i = 0; i < n; ++i) p[i] = rnd() * scale;
  return p;
}
static uint16_t *hvec(size_t n) {   /* fp16 bit patterns of small normal numbers */
  uint16_t *p = (uint16_t *)malloc(n * sizeof(uint16_t));
  for (size_t i = 0; i < n; ++i) p[i] = (uint16_t)(0x2000u + (rng_state = rng_state * 1664525u + 1013904223u) % 0x0c00u) |
                                        (uint16_t)((rng_state >> 20 & 1u) << 15);
  return p;
}
static real *rvec(size_t n) {
  real *p = (real *)malloc(n * sizeof(real));
  for (size_t i = 0; i < n; ++i) p[i] = (real)rnd();
  return p;
}
#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

static int run_model(int dtype, int n_layers, int H, int dh, int F, int V, int max_seq, int n_steps) {
  const int d = H * dh;
  oracle_config cfg = {n_layers, d, H, dh, F, V, max_seq, 10000.0f, 1e-5f};
  oracle_layer *layers = (oracle_layer *)malloc(sizeof(oracle_layer) * (size_t)n_layers);
  void **keep = (void **)malloc(sizeof(void *) * (size_t)(n_layers * 9 + 3));
  int nk = 0;
#define W(n) (keep[nk] = (dtype == ORACLE_DT_F16 ? (void *)hvec(n) : (void *)fvec(n, 0.05f)), keep[nk++])
  for (int l = 0; l < n_layers; ++l) {
    layers[l].attn_norm = W((size_t)d); layers[l].wq = W((size_t)d * d); layers[l].wk = W((size_t)d * d);
    layers[l].wv = W((size_t)d * d); layers[l].wo = W((size_t)d * d); layers[l].ffn_norm = W((size_t)d);
    layers[l].w_gate = W((size_t)F * d); layers[l].w_up = W((size_t)F * d); layers[l].w_down = W((size_t)d * F);
  }
  oracle_weights w;
  memset(&w, 0, sizeof w);
  w.tok_emb = W((size_t)V * d); w.final_norm = W((size_t)d); w.lm_head = W((size_t)V * d);
#undef W
  w.layers = layers;
  w.dtype = dtype;
  oracle_model *m = oracle_model_new(&cfg, &w);
  CHECK(m != NULL);
  real *logits = (real *)malloc(sizeof(real) * (size_t)V), *hidden = (real *)malloc(sizeof(real) * (size_t)d);
  int tok = 1 % V;
  for (int i = 0; i < n_steps; ++i) {
    tok = oracle_model_step(m, tok, logits, hidden);
    CHECK(tok >= 0 && tok < V && oracle_model_pos(m) == i + 1);
    for (int j = 0; j < V; ++j) CHECK(isfinite((double)logits[j]));
  }
  if (n_steps == max_seq) CHECK(oracle_model_step(m, 0, logits, hidden) < 0);   /* cache full: refused, nothing written */
  CHECK(oracle_model_step(m, V, logits, hidden) < 0 && oracle_model_step(m, -1, logits, hidden) < 0);
  for (int l = 0; l < n_layers; ++l)
    for (int which = 0; which < 2; ++which) {
      const real *kv = oracle_model_kv(m, l, which);
      real s = 0;
      for (size_t j = 0; j < (size_t)oracle_model_pos(m) * (size_t)d; ++j) s += kv[j];
      CHECK(isfinite((double)s));
    }
  oracle_model_reset(m);
  CHECK(oracle_model_pos(m) == 0 && oracle_model_step(m, 0, logits, hidden) >= 0);
  oracle_model_free(m);
  free(logits); free(hidden);
  for (int i = 0; i < nk; ++i) free(keep[i]);
  free(keep); free(layers);
  return 0;
}

int main(void) {
  CHECK(oracle_real_bytes() == (int)sizeof(real));
  for (uint32_t h = 0; h < 65536u; ++h) (void)oracle_half_to_float((uint16_t)h);
  /* operators on exact-size buffers, odd sizes */
  for (int n = 1; n <= 67; n += 11) {
    real *x = rvec((size_t)n), *out = rvec((size_t)n);
    float *g = fvec((size_t)n, 1.0f);
    uint16_t *gh = hvec((size_t)n);
    oracle_rmsnorm(x, g, ORACLE_DT_F32, n, 1e-5f, out);
    oracle_rmsnorm(x, gh, ORACLE_DT_F16, n, 1e-5f, out);
    real *m = rvec((size_t)n);
    oracle_swiglu(x, out, n, m);
    CHECK(oracle_argmax(m, n) >= 0 && oracle_argmax(m, n) < n);
    for (int rows = 1; rows <= 9; rows += 4) {
      float *W = fvec((size_t)rows * n, 1.0f);
      uint16_t *Wh = hvec((size_t)rows * n);
      real *y = rvec((size_t)rows);
      oracle_matvec(W, ORACLE_DT_F32, rows, n, x, y);
      oracle_matvec(Wh, ORACLE_DT_F16, rows, n, x, y);
      free(W); free(Wh); free(y);
    }
    free(x); free(out); free(g); free(gh); free(m);
  }
  for (int dh = 2; dh <= 128; dh *= 4)
    for (int H = 1; H <= 3; ++H) {
      real *v = rvec((size_t)H * dh);
      oracle_rope(v, H, dh, 0, 10000.0f);
      oracle_rope(v, H, dh, 4095, 10000.0f);
      free(v);
      for (int nk = 1; nk <= 33; nk += 16) {
        real *q = rvec((size_t)dh), *K = rvec((size_t)nk * dh), *V = rvec((size_t)nk * dh);
        real *o = rvec((size_t)dh), *wts = rvec((size_t)nk);
        oracle_attention_head(q, K, V, nk, dh, dh, o, wts);
        real sum = 0;
        for (int u = 0; u < nk; ++u) sum += wts[u];
        CHECK(fabs((double)sum - 1.0) < 1e-4);
        free(q); free(K); free(V); free(o); free(wts);
      }
    }
  /* whole model: the tiny configuration, fp32 and fp16 weights, decoded until the cache is full */
  if (run_model(ORACLE_DT_F32, 2, 4, 64, 688, 1024, 26, 26)) return 1;
  if (run_model(ORACLE_DT_F16, 2, 4, 64, 688, 1024, 26, 26)) return 1;
  if (run_model(ORACLE_DT_F16, 1, 3, 128, 1000, 501, 7, 5)) return 1;     /* ragged sizes */
  if (run_model(ORACLE_DT_F32, 1, 1, 2, 8, 3, 2, 2)) return 1;            /* smallest everything */
  printf("oracle sanitizer run ok (%d-byte reals)\n", (int)sizeof(real));
  return 0;
}
