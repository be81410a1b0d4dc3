/*
 * CPU ORACLE -- TEST INFRASTRUCTURE ONLY (see spec_oracle.h).
 * Plain C, one left-to-right loop per reduction, arithmetic in `real`.
 * OpenMP, where present, only distributes independent output elements over
 * threads; no reduction is split, so results do not depend on thread count.
 */
#include "spec_oracle.h"
#include <math.h>
#include <stdlib.h>
#include <string.h>

#define R_EXP(x)  ((real)exp((double)(x)))
#define R_SQRT(x) ((real)sqrt((double)(x)))

int orc_real_bytes(void) { return (int)sizeof(real); }

/* ------------------------------------------------------------------ widening */

static float bits_to_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/* bf16 is the upper half of an IEEE binary32. */
static float bf16_to_f32(uint16_t h) { return bits_to_f32((uint32_t)h << 16); }

/* IEEE binary16 -> binary32, exact. */
static float f16_to_f32(uint16_t h) {
  uint32_t sign = (uint32_t)(h >> 15) << 31;
  int32_t  e = (h >> 10) & 0x1f;
  uint32_t m = h & 0x3ff;
  if (e == 0) {
    if (m == 0) return bits_to_f32(sign);
    /* subnormal: value = m * 2^-24 */
    float v = (float)m * (1.0f / 16777216.0f);
    return sign ? -v : v;
  }
  if (e == 31) return bits_to_f32(sign | 0x7f800000u | (m << 13));
  return bits_to_f32(sign | ((uint32_t)(e - 15 + 127) << 23) | (m << 13));
}

static inline real w_at(const void *p, int wdtype, int64_t i) {
  switch (wdtype) {
    case ORC_W_F32:  return (real)((const float *)p)[i];
    case ORC_W_BF16: return (real)bf16_to_f32(((const uint16_t *)p)[i]);
    default:         return (real)f16_to_f32(((const uint16_t *)p)[i]);
  }
}

void orc_widen(const void *src, int wdtype, int64_t n, real *dst) {
  for (int64_t i = 0; i < n; ++i) dst[i] = w_at(src, wdtype, i);
}

/* ------------------------------------------------------ elementary operations */

/* y[m][n] = sum_k x[m][k] * W[n][k] (+ bias[n]); the weight matrices the paper
   says dominate the step (Sec. 1, Sec. 3.3).                                   */
void orc_linear(const real *x, int M, int K, const void *W, const void *bias, int wdtype, int N, real *y) {
#pragma omp parallel for schedule(static)
  for (int n = 0; n < N; ++n) {
    for (int m = 0; m < M; ++m) {
      real acc = 0;
      for (int k = 0; k < K; ++k) acc += x[(int64_t)m * K + k] * w_at(W, wdtype, (int64_t)n * K + k);
      if (bias) acc += w_at(bias, wdtype, n);
      y[(int64_t)m * N + n] = acc;
    }
  }
}

/* RMSNorm (LLaMA-shape models): y = x / sqrt(mean(x^2) + eps) * gain. */
void orc_rmsnorm(const real *x, int M, int d, const void *gain, int wdtype, double eps, real *y) {
  for (int m = 0; m < M; ++m) {
    real ss = 0;
    for (int i = 0; i < d; ++i) ss += x[(int64_t)m * d + i] * x[(int64_t)m * d + i];
    real inv = (real)1 / R_SQRT(ss / (real)d + (real)eps);
    for (int i = 0; i < d; ++i) y[(int64_t)m * d + i] = x[(int64_t)m * d + i] * inv * w_at(gain, wdtype, i);
  }
}

/* LayerNorm (OPT-shape models): y = (x - mean) / sqrt(var + eps) * gain + bias. */
void orc_layernorm(const real *x, int M, int d, const void *gain, const void *bias, int wdtype, double eps, real *y) {
  for (int m = 0; m < M; ++m) {
    real mean = 0;
    for (int i = 0; i < d; ++i) mean += x[(int64_t)m * d + i];
    mean /= (real)d;
    real var = 0;
    for (int i = 0; i < d; ++i) { real c = x[(int64_t)m * d + i] - mean; var += c * c; }
    var /= (real)d;
    real inv = (real)1 / R_SQRT(var + (real)eps);
    for (int i = 0; i < d; ++i)
      y[(int64_t)m * d + i] = (x[(int64_t)m * d + i] - mean) * inv * w_at(gain, wdtype, i) + w_at(bias, wdtype, i);
  }
}

/* Rotary embedding, rotate-half pairing: within each head, element i pairs with
   i + hd/2 and the pair turns by pos * theta^(-2i/hd).                        */
void orc_rope(real *x, int n_heads, int hd, int pos, double theta) {
  int half = hd / 2;
  for (int h = 0; h < n_heads; ++h) {
    real *v = x + (int64_t)h * hd;
    for (int i = 0; i < half; ++i) {
      double ang = (double)pos * pow(theta, -2.0 * (double)i / (double)hd);
      real c = (real)cos(ang), s = (real)sin(ang);
      real a = v[i], b = v[i + half];
      v[i]        = a * c - b * s;
      v[i + half] = b * c + a * s;
    }
  }
}

/* One query row against n_keys cached rows, every head on its own slice:
   out = softmax(q K^T / sqrt(hd)) V.  Kc, Vc: [n_keys][n_heads*hd].           */
void orc_attention(const real *q, int n_heads, int hd, const real *Kc, const real *Vc, int n_keys, real *out) {
  int d = n_heads * hd;
  real scale = (real)1 / R_SQRT((real)hd);
  real *p = (real *)malloc(sizeof(real) * (size_t)n_keys);
  for (int h = 0; h < n_heads; ++h) {
    const real *qh = q + (int64_t)h * hd;
    real mx = 0;
    for (int j = 0; j < n_keys; ++j) {
      const real *kj = Kc + (int64_t)j * d + (int64_t)h * hd;
      real dot = 0;
      for (int i = 0; i < hd; ++i) dot += qh[i] * kj[i];
      p[j] = dot * scale;
      if (j == 0 || p[j] > mx) mx = p[j];
    }
    real sum = 0;
    for (int j = 0; j < n_keys; ++j) { p[j] = R_EXP(p[j] - mx); sum += p[j]; }
    for (int i = 0; i < hd; ++i) {
      real acc = 0;
      for (int j = 0; j < n_keys; ++j) acc += p[j] * Vc[(int64_t)j * d + (int64_t)h * hd + i];
      out[(int64_t)h * hd + i] = acc / sum;
    }
  }
  free(p);
}

/* SwiGLU gating: silu(g) * u with silu(g) = g / (1 + exp(-g)). */
void orc_swiglu(const real *gate, const real *up, int64_t n, real *out) {
  for (int64_t i = 0; i < n; ++i) out[i] = gate[i] / ((real)1 + R_EXP(-gate[i])) * up[i];
}

void orc_relu(const real *x, int64_t n, real *out) {
  for (int64_t i = 0; i < n; ++i) out[i] = x[i] > 0 ? x[i] : (real)0;
}

/* Greedy choice (Alg. 1 reads "argmin"; the caption and Sec. 2 say highest
   probability, so this is the arg-MAX); lowest index wins a tie.              */
int orc_argmax(const real *v, int n) {
  int best = 0;
  for (int i = 1; i < n; ++i) if (v[i] > v[best]) best = i;
  return best;
}

/* ------------------------------------------------------------------- model */

struct orc_model {
  orc_desc d;
  orc_weights w;
  const void **layers;
};

struct orc_cache {
  int n_layers, d, L_max;
  real *k, *v; /* [n_layers][L_max][d] */
};

orc_model *orc_model_create(const orc_desc *desc, const orc_weights *w) {
  if (!desc || !w || desc->n_layers < 0 || desc->d_model <= 0 || desc->n_heads <= 0 ||
      desc->d_model % desc->n_heads != 0 || (desc->d_model / desc->n_heads) % 2 != 0) return NULL;
  orc_model *m = (orc_model *)calloc(1, sizeof(orc_model));
  m->d = *desc;
  m->w = *w;
  size_t n = (size_t)desc->n_layers * ORC_T_COUNT;
  m->layers = (const void **)malloc(sizeof(void *) * (n ? n : 1));
  for (size_t i = 0; i < n; ++i) m->layers[i] = w->layers[i];
  m->w.layers = m->layers;
  return m;
}

void orc_model_destroy(orc_model *m) { if (m) { free(m->layers); free(m); } }

orc_cache *orc_cache_create(const orc_model *m, int L_max) {
  orc_cache *c = (orc_cache *)calloc(1, sizeof(orc_cache));
  c->n_layers = m->d.n_layers; c->d = m->d.d_model; c->L_max = L_max;
  size_t n = (size_t)c->n_layers * (size_t)L_max * (size_t)c->d;
  c->k = (real *)calloc(n ? n : 1, sizeof(real));
  c->v = (real *)calloc(n ? n : 1, sizeof(real));
  return c;
}

void orc_cache_destroy(orc_cache *c) { if (c) { free(c->k); free(c->v); free(c); } }
real *orc_cache_k(orc_cache *c, int layer) { return c->k + (size_t)layer * c->L_max * c->d; }
real *orc_cache_v(orc_cache *c, int layer) { return c->v + (size_t)layer * c->L_max * c->d; }

static void norm_rows(const orc_model *m, const real *x, int M, const void *g, const void *b, real *y) {
  if (m->d.norm_kind == ORC_NORM_RMS) orc_rmsnorm(x, M, m->d.d_model, g, m->w.wdtype, m->d.norm_eps, y);
  else orc_layernorm(x, M, m->d.d_model, g, b, m->w.wdtype, m->d.norm_eps, y);
}

/* The verification forward of Alg. 1 (the call LLM(S, t_1..t_s, kv)), and
   equally the draft model's decode step: q new tokens of one sequence against
   that sequence's cache, causal among the new tokens.                         */
int orc_forward(const orc_model *m, orc_cache *c, const int32_t *tokens, int q, int start_pos, real *logits) {
  const orc_desc *D = &m->d;
  const int d = D->d_model, H = D->n_heads, hd = d / H, f = D->d_ffn, wt = m->w.wdtype;
  if (q <= 0) return 0;
  if (start_pos < 0 || start_pos + q > c->L_max) return -1;
  if (D->pos_kind == ORC_POS_LEARNED && start_pos + q > D->max_pos) return -1;
  for (int i = 0; i < q; ++i) if (tokens[i] < 0 || tokens[i] >= D->vocab) return -2;

  size_t qd = (size_t)q * d, qf = (size_t)q * f;
  real *h  = (real *)malloc(sizeof(real) * qd);
  real *x  = (real *)malloc(sizeof(real) * qd);
  real *qv = (real *)malloc(sizeof(real) * qd);
  real *kv = (real *)malloc(sizeof(real) * qd);
  real *vv = (real *)malloc(sizeof(real) * qd);
  real *at = (real *)malloc(sizeof(real) * qd);
  real *o  = (real *)malloc(sizeof(real) * qd);
  real *g  = (real *)malloc(sizeof(real) * qf);
  real *u  = (real *)malloc(sizeof(real) * qf);

  for (int i = 0; i < q; ++i)
    for (int j = 0; j < d; ++j) {
      real e = w_at(m->w.tok_emb, wt, (int64_t)tokens[i] * d + j);
      if (D->pos_kind == ORC_POS_LEARNED) e += w_at(m->w.pos_emb, wt, (int64_t)(start_pos + i) * d + j);
      h[(size_t)i * d + j] = e;
    }

  for (int L = 0; L < D->n_layers; ++L) {
    const void *const *T = m->layers + (size_t)L * ORC_T_COUNT;
    const int hb = D->has_bias;
    norm_rows(m, h, q, T[ORC_T_ATTN_NORM_W], T[ORC_T_ATTN_NORM_B], x);
    orc_linear(x, q, d, T[ORC_T_WQ], hb ? T[ORC_T_BQ] : NULL, wt, d, qv);
    orc_linear(x, q, d, T[ORC_T_WK], hb ? T[ORC_T_BK] : NULL, wt, d, kv);
    orc_linear(x, q, d, T[ORC_T_WV], hb ? T[ORC_T_BV] : NULL, wt, d, vv);
    real *Kc = orc_cache_k(c, L), *Vc = orc_cache_v(c, L);
    for (int i = 0; i < q; ++i) {
      int pos = start_pos + i;
      if (D->pos_kind == ORC_POS_ROPE) {
        orc_rope(qv + (size_t)i * d, H, hd, pos, D->rope_theta);
        orc_rope(kv + (size_t)i * d, H, hd, pos, D->rope_theta);
      }
      memcpy(Kc + (size_t)pos * d, kv + (size_t)i * d, sizeof(real) * d);
      memcpy(Vc + (size_t)pos * d, vv + (size_t)i * d, sizeof(real) * d);
    }
    for (int i = 0; i < q; ++i)
      orc_attention(qv + (size_t)i * d, H, hd, Kc, Vc, start_pos + i + 1, at + (size_t)i * d);
    orc_linear(at, q, d, T[ORC_T_WO], hb ? T[ORC_T_BO] : NULL, wt, d, o);
    for (size_t i = 0; i < qd; ++i) h[i] += o[i];

    norm_rows(m, h, q, T[ORC_T_FFN_NORM_W], T[ORC_T_FFN_NORM_B], x);
    if (D->ffn_kind == ORC_FFN_SWIGLU) {
      orc_linear(x, q, d, T[ORC_T_W1], NULL, wt, f, g);
      orc_linear(x, q, d, T[ORC_T_W3], NULL, wt, f, u);
      orc_swiglu(g, u, (int64_t)qf, g);
    } else {
      orc_linear(x, q, d, T[ORC_T_W1], hb ? T[ORC_T_B1] : NULL, wt, f, g);
      orc_relu(g, (int64_t)qf, g);
    }
    orc_linear(g, q, f, T[ORC_T_W2], (hb && D->ffn_kind == ORC_FFN_RELU) ? T[ORC_T_B2] : NULL, wt, d, o);
    for (size_t i = 0; i < qd; ++i) h[i] += o[i];
  }

  if (logits) {
    norm_rows(m, h, q, m->w.final_norm_w, m->w.final_norm_b, x);
    orc_linear(x, q, d, m->w.lm_head, NULL, wt, D->vocab, logits);
  }
  free(h); free(x); free(qv); free(kv); free(vv); free(at); free(o); free(g); free(u);
  return 0;
}

/* ------------------------------------------------------------------ method */

/* Sec. 2: a proposal survives only while every earlier proposal survived; the
   target then adds its own token after the last survivor (a correction if
   l < s, a look-ahead if l = s).                                              */
int orc_accept(const int32_t *t, int s, const int32_t *a, int32_t *emitted) {
  int l = 0;
  while (l < s && t[l] == a[l]) ++l;
  for (int i = 0; i < l; ++i) emitted[i] = t[i];
  emitted[l] = a[l];
  return l;
}

int orc_greedy(const orc_model *tgt, const int32_t *prompt, int P, int N, int L_max, int32_t *out) {
  if (P < 1 || P + N > L_max + 1) return -1;
  orc_cache *c = orc_cache_create(tgt, L_max);
  real *logits = (real *)malloc(sizeof(real) * (size_t)tgt->d.vocab);
  int rc = 0;
  if (P > 1) rc = orc_forward(tgt, c, prompt, P - 1, 0, NULL);
  int32_t cur = prompt[P - 1];
  for (int i = 0; i < N && rc == 0; ++i) {
    rc = orc_forward(tgt, c, &cur, 1, P - 1 + i, logits);
    if (rc) break;
    cur = orc_argmax(logits, tgt->d.vocab);
    out[i] = cur;
  }
  free(logits); orc_cache_destroy(c);
  return rc;
}

int orc_spec_generate(const orc_model *tgt, const orc_model *drf, const int32_t *prompt, int P, int N,
                      int s, int proposal_mode, const int32_t *prop_table, int L_max,
                      int32_t *out, int32_t *stats_l, int32_t *rounds) {
  if (P < 1 || s < 0 || P + N + s > L_max) return -1;
  if (proposal_mode == 0 && s > 0 && !drf) return -1;
  if (proposal_mode == 1 && s > 0 && !prop_table) return -1;
  const int V = tgt->d.vocab;
  int32_t *S = (int32_t *)malloc(sizeof(int32_t) * (size_t)(P + N + s + 1));
  memcpy(S, prompt, sizeof(int32_t) * (size_t)P);
  int32_t *t = (int32_t *)malloc(sizeof(int32_t) * (size_t)(s + 1));
  int32_t *a = (int32_t *)malloc(sizeof(int32_t) * (size_t)(s + 1));
  int32_t *in = (int32_t *)malloc(sizeof(int32_t) * (size_t)(s + 1));
  int32_t *em = (int32_t *)malloc(sizeof(int32_t) * (size_t)(s + 1));
  real *lt = (real *)malloc(sizeof(real) * (size_t)(s + 1) * V);
  real *ld = drf ? (real *)malloc(sizeof(real) * (size_t)(s + 2) * drf->d.vocab) : NULL;
  orc_cache *ct = orc_cache_create(tgt, L_max);
  orc_cache *cd = drf ? orc_cache_create(drf, L_max) : NULL;
  int rc = 0, n = P, gen = 0, nr = 0;
  int kvD = P - 1; /* draft cache holds positions 0..kvD-1 */

  if (P > 1) {
    rc = orc_forward(tgt, ct, prompt, P - 1, 0, NULL);
    if (!rc && drf) rc = orc_forward(drf, cd, prompt, P - 1, 0, NULL);
  }
  while (!rc && gen < N) {
    /* speculate(S, kv_SSM, s): s sequential greedy steps of the small model */
    for (int j = 1; j <= s && !rc; ++j) {
      int td = -1;
      if (drf) {
        if (j == 1) {
          int cnt = n - kvD; /* committed tokens the draft has not read yet */
          rc = orc_forward(drf, cd, S + kvD, cnt, kvD, ld);
          if (!rc) td = orc_argmax(ld + (size_t)(cnt - 1) * drf->d.vocab, drf->d.vocab);
        } else {
          rc = orc_forward(drf, cd, &t[j - 2], 1, n + j - 2, ld);
          if (!rc) td = orc_argmax(ld, drf->d.vocab);
        }
      }
      t[j - 1] = (proposal_mode == 0) ? td : prop_table[n + j - 1];
    }
    if (rc) break;
    /* LLM(S, t_1..t_s, kv_LLM): last committed token plus the s proposals */
    in[0] = S[n - 1];
    for (int j = 0; j < s; ++j) in[j + 1] = t[j];
    rc = orc_forward(tgt, ct, in, s + 1, n - 1, lt);
    if (rc) break;
    for (int i = 0; i <= s; ++i) a[i] = orc_argmax(lt + (size_t)i * V, V);
    int l = orc_accept(t, s, a, em);
    int take = l + 1;
    if (gen + take > N) take = N - gen;
    for (int i = 0; i < take; ++i) { S[n + i] = em[i]; out[gen + i] = em[i]; }
    if (stats_l) stats_l[nr] = l;
    ++nr;
    /* rejected positions are dropped: only lengths move (Sec. 3.1) */
    if (s > 0 && drf) kvD = n + (l < s - 1 ? l : s - 1);
    n += take; gen += take;
    if (kvD > n - 1) kvD = n - 1;
  }
  if (rounds) *rounds = nr;
  free(S); free(t); free(a); free(in); free(em); free(lt); free(ld);
  orc_cache_destroy(ct); orc_cache_destroy(cd);
  return rc;
}

/* ------------------------------------------------------ adaptive policy (Sec. 4) */

void orc_lut_build(const double *lat, int nB, int nS, double rel_eps, int32_t *lut) {
  for (int b = 0; b < nB; ++b) {
    const double *row = lat + (size_t)b * nS;
    double best = row[0];
    for (int s = 1; s < nS; ++s) if (row[s] < best) best = row[s];
    int pick = 0;
    while (row[pick] > best * (1.0 + rel_eps)) ++pick; /* smallest s within eps of the minimum */
    lut[b] = pick;
  }
}

int orc_lut_lookup(const int32_t *profiled_B, const int32_t *lut, int nB, int B) {
  /* profiled_B ascending */
  if (B <= profiled_B[0]) return lut[0];
  for (int i = 0; i < nB; ++i) if (profiled_B[i] == B) return lut[i];
  if (B > profiled_B[nB - 1]) return lut[nB - 1];
  int hi = 0;
  while (profiled_B[hi] < B) ++hi;
  int lo = hi - 1;
  return lut[lo] < lut[hi] ? lut[lo] : lut[hi];
}

double orc_l_estimate(const int32_t *l_i, int n, int s) {
  double acc = 0;
  for (int i = 0; i < n; ++i) acc += (double)(l_i[i] < s ? l_i[i] : s);
  return acc / (double)n;
}

double orc_time_model(double N, double tL, double tS, double s, double l_of_s) {
  return N * tL / (l_of_s + 1.0) + N * s * tS / (l_of_s + 1.0);
}
