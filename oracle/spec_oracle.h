/*
 * CPU ORACLE -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct implementation of batched greedy
 * speculative decoding (Alg. 1 of the paper, Sec. 2 "Speculative Decoding",
 * Sec. 3.1 for the batched form, Sec. 4 for the adaptive look-up table).
 * It exists to check the GPU library; nothing in the product path may call
 * it.  It shares no code with the GPU library.
 *
 * Built twice from this one source: ORC_REAL=float (the fp32 oracle) and
 * ORC_REAL=double (the fp64 oracle used as parity reference).
 *
 * Parameters arrive as fp32, bf16 bits or fp16 bits (wdtype) and are widened
 * exactly; every arithmetic step runs in ORC_REAL.  No blocking, no fusion,
 * no reordering: every reduction is a left-to-right loop.
 *
 * Parity pins (tests/test_oracle_*.py): the decoder forward is pinned against
 * the HuggingFace LLaMA / OPT implementations (the model layer the paper's
 * prototype ran on, Sec. 3.1), RoPE/softmax/norms against closed forms, the
 * speculative loop against plain autoregressive greedy decoding (the defining
 * invariant, Sec. 2), its draft-cache bookkeeping by running it with the target's
 * own weights as the draft (every round must then accept all s proposals, which
 * a wrong cache length or a mis-sized first draft step breaks), acceptance
 * against hand-worked cases, acceptance
 * statistics against Eq. 6 in closed form, the LUT rule against enumerated
 * cases of Sec. 4.  Parity unpinned: the fitted constants 0.9 and 0.548 of
 * Eq. 5 (they need the paper's trained models and dataset); they are not
 * implemented.
 */
#ifndef SPEC_ORACLE_H
#define SPEC_ORACLE_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

#ifndef ORC_REAL
#define ORC_REAL double
#endif
typedef ORC_REAL real;

enum { ORC_W_F32 = 0, ORC_W_BF16 = 1, ORC_W_F16 = 2 };
enum { ORC_FFN_SWIGLU = 0, ORC_FFN_RELU = 1 };
enum { ORC_NORM_RMS = 0, ORC_NORM_LAYER = 1 };
enum { ORC_POS_ROPE = 0, ORC_POS_LEARNED = 1 };

/* Per-layer tensor slots; every matrix is row-major [out][in]. */
enum {
  ORC_T_ATTN_NORM_W = 0, ORC_T_ATTN_NORM_B,
  ORC_T_WQ, ORC_T_BQ, ORC_T_WK, ORC_T_BK, ORC_T_WV, ORC_T_BV, ORC_T_WO, ORC_T_BO,
  ORC_T_FFN_NORM_W, ORC_T_FFN_NORM_B,
  ORC_T_W1, ORC_T_B1,      /* SwiGLU gate [f][d]  | ReLU fc1 [f][d] */
  ORC_T_W3,                /* SwiGLU up   [f][d]  | unused          */
  ORC_T_W2, ORC_T_B2,      /* down / fc2  [d][f]                    */
  ORC_T_COUNT
};

typedef struct {
  int32_t n_layers, d_model, n_heads, d_ffn, vocab, max_pos;
  int32_t ffn_kind, norm_kind, pos_kind, has_bias;
  double norm_eps, rope_theta;
} orc_desc;

typedef struct {
  int32_t wdtype;
  const void *tok_emb;      /* [vocab][d] */
  const void *pos_emb;      /* [max_pos][d], learned positions only */
  const void *final_norm_w; /* [d] */
  const void *final_norm_b; /* [d], LayerNorm only */
  const void *lm_head;      /* [vocab][d] */
  const void *const *layers; /* n_layers * ORC_T_COUNT pointers */
} orc_weights;

typedef struct orc_model orc_model;
typedef struct orc_cache orc_cache;

int  orc_real_bytes(void);

/* ---- elementary operations (each usable alone by the per-kernel tests) ---- */
void orc_widen(const void *src, int wdtype, int64_t n, real *dst);
void orc_linear(const real *x, int M, int K, const void *W, const void *bias, int wdtype, int N, real *y);
void orc_rmsnorm(const real *x, int M, int d, const void *gain, int wdtype, double eps, real *y);
void orc_layernorm(const real *x, int M, int d, const void *gain, const void *bias, int wdtype, double eps, real *y);
void orc_rope(real *x, int n_heads, int hd, int pos, double theta);
void orc_attention(const real *q, int n_heads, int hd, const real *Kc, const real *Vc, int n_keys, real *out);
void orc_swiglu(const real *gate, const real *up, int64_t n, real *out);
void orc_relu(const real *x, int64_t n, real *out);
int  orc_argmax(const real *v, int n);

/* ---- decoder model with a per-sequence KV cache ---- */
orc_model *orc_model_create(const orc_desc *desc, const orc_weights *w);
void       orc_model_destroy(orc_model *m);
orc_cache *orc_cache_create(const orc_model *m, int L_max);
void       orc_cache_destroy(orc_cache *c);
/* direct access for tests that pre-fill a cache: K/V rows are [L_max][d_model] per layer */
real      *orc_cache_k(orc_cache *c, int layer);
real      *orc_cache_v(orc_cache *c, int layer);

/* Feed q tokens at positions start_pos .. start_pos+q-1; keys 0..start_pos-1
   come from the cache; the q new K/V rows are written at their positions
   (overwriting whatever was there).  logits: [q][vocab] or NULL.            */
int orc_forward(const orc_model *m, orc_cache *c, const int32_t *tokens, int q, int start_pos, real *logits);

/* ---- the method ---- */
/* Acceptance rule (Sec. 2; Alg. 1): l = number of leading proposals equal to the
   target's greedy token; emitted = t_1..t_l, a_l.  Returns l.                 */
int orc_accept(const int32_t *t, int s, const int32_t *a, int32_t *emitted);

/* Plain autoregressive greedy decoding: the definition every speculative
   variant must reproduce.  out: [N].                                          */
int orc_greedy(const orc_model *tgt, const int32_t *prompt, int P, int N, int L_max, int32_t *out);

/* One sequence of Alg. 1.  proposal_mode 0: the draft model's greedy tokens;
   1: proposals read from prop_table[pos] for absolute position pos (the draft
   model, if given, still runs and ingests those tokens).  out: [N].
   stats_l: accepted count per round (capacity N), *rounds = number of rounds. */
int orc_spec_generate(const orc_model *tgt, const orc_model *drf, const int32_t *prompt, int P, int N,
                      int s, int proposal_mode, const int32_t *prop_table, int L_max,
                      int32_t *out, int32_t *stats_l, int32_t *rounds);

/* Sec. 4: LUT[B_i] = argmin_s of the measured per-token latency (ties within
   rel_eps resolved towards the smaller s); lookup rule for un-profiled B.     */
void orc_lut_build(const double *lat, int nB, int nS, double rel_eps, int32_t *lut);
int  orc_lut_lookup(const int32_t *profiled_B, const int32_t *lut, int nB, int B);

/* Eq. 4: l(s) ~ (1/n) sum_i min(l_i, s).  Eq. 7: per-token time model.        */
double orc_l_estimate(const int32_t *l_i, int n, int s);
double orc_time_model(double N, double tL, double tS, double s, double l_of_s);

#ifdef __cplusplus
}
#endif
#endif
