// Host runtime behind the C ABI of include/spec.h: argument validation, workspace
// carving, launch sequencing of one speculative-decoding round (Alg. 1), the profiling
// grid and the batch-size -> speculation-length table (Sec. 4).
#include "spec_internal.h"
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>

using namespace spec;


static thread_local std::string g_err;

static int fail(spec_ctx *c, int code, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  if (c) c->err = buf;
  return code;
}
// for the entry points that live in other files and have no context
int spec::fail_noctx(int code, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}
#define HIPCHK(c, call)                                                                      \
  do {                                                                                       \
    hipError_t e_ = (call);                                                                  \
    if (e_ != hipSuccess) return fail((c), SPEC_ERR_HIP, "%s: %s", #call, hipGetErrorString(e_)); \
  } while (0)

extern "C" const char *spec_last_error(const spec_ctx *c) { return c ? c->err.c_str() : g_err.c_str(); }

// ------------------------------------------------------------------ sizing
static size_t al256(size_t b) { return (b + 255) & ~(size_t)255; }
constexpr int PREFILL_CHUNK = 8;
constexpr int Q_LIMIT = 16;  // rows per sequence in one pass (attention query tile)

static int check_model(const spec_model_desc *d, const char *who, int dtype) {
  if (d->n_layers < 1 || d->d_model < 2 || d->n_heads < 1 || d->d_ffn < 1 || d->vocab < 1)
    return fail(nullptr, SPEC_ERR_INVALID_ARG, "%s: n_layers, d_model, n_heads, d_ffn, vocab must be positive", who);
  if (d->d_model % d->n_heads != 0 || (d->d_model / d->n_heads) % 2 != 0)
    return fail(nullptr, SPEC_ERR_INVALID_ARG, "%s: d_model must be a multiple of n_heads with an even head_dim", who);
  if (d->d_model % 4 != 0 || d->d_model > 8192)
    return fail(nullptr, SPEC_ERR_UNSUPPORTED, "%s: d_model must be a multiple of 4 and at most 8192", who);
  if (d->ffn_kind != SPEC_FFN_SWIGLU && d->ffn_kind != SPEC_FFN_RELU)
    return fail(nullptr, SPEC_ERR_INVALID_ARG, "%s: unknown ffn_kind %d", who, d->ffn_kind);
  if (d->norm_kind != SPEC_NORM_RMS && d->norm_kind != SPEC_NORM_LAYER)
    return fail(nullptr, SPEC_ERR_INVALID_ARG, "%s: unknown norm_kind %d", who, d->norm_kind);
  if (d->pos_kind != SPEC_POS_ROPE && d->pos_kind != SPEC_POS_LEARNED)
    return fail(nullptr, SPEC_ERR_INVALID_ARG, "%s: unknown pos_kind %d", who, d->pos_kind);
  if (d->pos_kind == SPEC_POS_LEARNED && d->max_pos < 1)
    return fail(nullptr, SPEC_ERR_INVALID_ARG, "%s: learned positions need max_pos >= 1", who);
  if (!(d->norm_eps > 0.f)) return fail(nullptr, SPEC_ERR_INVALID_ARG, "%s: norm_eps must be positive", who);
  if (d->pos_kind == SPEC_POS_ROPE && !(d->rope_theta > 1.f))
    return fail(nullptr, SPEC_ERR_INVALID_ARG, "%s: rope_theta must exceed 1", who);
  (void)dtype;
  return SPEC_OK;
}

static int check_run(const spec_run_desc *r) {
  if (r->dtype < SPEC_DTYPE_F32 || r->dtype > SPEC_DTYPE_F16)
    return fail(nullptr, SPEC_ERR_INVALID_ARG, "run: unknown dtype %d", r->dtype);
  if (r->B_max < 1 || r->B_max > 4096) return fail(nullptr, SPEC_ERR_INVALID_ARG, "run: B_max must be in 1..4096");
  if (r->s_max < 0 || r->s_max + 1 > Q_LIMIT)
    return fail(nullptr, SPEC_ERR_INVALID_ARG, "run: s_max must be in 0..%d", Q_LIMIT - 1);
  if (r->gen_max < 1) return fail(nullptr, SPEC_ERR_INVALID_ARG, "run: gen_max must be positive");
  if (r->L_max < r->gen_max + r->s_max + 1)
    return fail(nullptr, SPEC_ERR_INVALID_ARG, "run: L_max must be at least gen_max + s_max + 1");
  if (r->eos_id < -1) return fail(nullptr, SPEC_ERR_INVALID_ARG, "run: eos_id must be -1 (none) or a token id");
  if (r->proposal_mode != SPEC_PROPOSALS_DRAFT && r->proposal_mode != SPEC_PROPOSALS_EXTERNAL)
    return fail(nullptr, SPEC_ERR_INVALID_ARG, "run: unknown proposal_mode %d", r->proposal_mode);
  return SPEC_OK;
}

struct Sizes {
  int M_max, q_pass;
  size_t state, act, tgt_w, tgt_kv, drf_w, drf_kv, total;
  size_t kv_area_tgt, kv_area_drf;
  int L_pad;
};

static size_t packed_bytes(const spec_model_desc &d, int dtype, int L_max) {
  return fast_supported(d, dtype) ? fast_packed_bytes(d, dtype, L_max) : generic_packed_bytes(d, dtype);
}

static Sizes compute_sizes(const spec_model_desc *tgt, const spec_model_desc *drf, const spec_run_desc *run) {
  Sizes z{};
  const size_t e = dtype_bytes(run->dtype);
  z.q_pass = std::max(run->s_max + 1, PREFILL_CHUNK);
  z.M_max = run->B_max * z.q_pass;
  z.L_pad = (run->L_max + KV_LPAD - 1) / KV_LPAD * KV_LPAD;
  const size_t B = run->B_max, L = run->L_max, s = run->s_max, M = z.M_max;
  z.state = al256(B * L * 4) + 6 * al256(B * 4) + al256(B * std::max<size_t>(s, 1) * 4) + al256(B * (s + 1) * 4) +
            al256((s + 1) * 8) + al256(16) + al256(4);
  size_t d = tgt->d_model, f = tgt->d_ffn, V = tgt->vocab;
  size_t kf = tgt->ffn_kind == SPEC_FFN_SWIGLU ? 2 : 1;
  size_t wide = std::max(3 * d, kf * f);
  if (drf) {
    d = std::max<size_t>(d, drf->d_model);
    f = std::max<size_t>(f, drf->d_ffn);
    V = std::max<size_t>(V, drf->vocab);
    size_t kfd = drf->ffn_kind == SPEC_FFN_SWIGLU ? 2 : 1;
    wide = std::max(wide, std::max<size_t>(3 * (size_t)drf->d_model, kfd * drf->d_ffn));
  }
  const size_t Mp = (M + 15) / 16 * 16;  // fragment-order activation buffers hold whole 16-row tiles
  z.act = al256(M * d * 4) + 2 * al256(Mp * d * e) + al256(Mp * d * 4) + al256(Mp * f * e) + al256(M * wide * 4) + al256(M * V * 4) +
          3 * al256(M * 4);
  // matrix-core path: split-KV attention partials and per-strip arg-max partials
  const size_t NC = (size_t)attn_chunk_of((int)std::max<size_t>(L, 1) - 1) + 1, NTh = (V + 15) / 16;
  z.act += al256(M * d * NC * 4) + al256(M * (d / 64 + 1) * NC * 2 * 4) + 2 * al256(M * NTh * 4);
  if (M > 32) z.act += al256(8 * Mp * d * 4);  // k-slice sums of the split residual GEMMs
  z.act += 2 * al256(M * 4);  // 1 / rms (or 1 / std) and mean per row (folded norm)
  z.tgt_w = packed_bytes(*tgt, run->dtype, run->L_max);
  z.kv_area_tgt = B * (size_t)tgt->d_model * z.L_pad;
  z.tgt_kv = 2 * al256((size_t)tgt->n_layers * z.kv_area_tgt * e);
  if (drf) {
    z.drf_w = packed_bytes(*drf, run->dtype, run->L_max);
    z.kv_area_drf = B * (size_t)drf->d_model * z.L_pad;
    z.drf_kv = 2 * al256((size_t)drf->n_layers * z.kv_area_drf * e);
  }
  z.total = z.state + z.act + z.tgt_w + z.tgt_kv + z.drf_w + z.drf_kv;
  return z;
}

extern "C" int spec_workspace_bytes(const spec_model_desc *tgt, const spec_model_desc *drf, const spec_run_desc *run,
                                    size_t *bytes) {
  if (!tgt || !run || !bytes) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_workspace_bytes: null argument");
  int rc = check_run(run);
  if (rc) return rc;
  if ((rc = check_model(tgt, "target", run->dtype))) return rc;
  if (drf && (rc = check_model(drf, "draft", run->dtype))) return rc;
  if (drf && drf->vocab != tgt->vocab)
    return fail(nullptr, SPEC_ERR_INVALID_ARG, "draft and target must share one vocabulary");
  if (run->eos_id >= tgt->vocab)
    return fail(nullptr, SPEC_ERR_INVALID_ARG, "run: eos_id %d outside the vocabulary (%d tokens)", run->eos_id, tgt->vocab);
  *bytes = compute_sizes(tgt, drf, run).total;
  return SPEC_OK;
}

// ------------------------------------------------------------------ init
static int check_weights(const spec_model_desc *d, const spec_weights *w, const char *who) {
  if (!w->d_tok_emb || !w->d_final_norm_w || !w->d_lm_head || !w->layer_tensors)
    return fail(nullptr, SPEC_ERR_INVALID_ARG, "%s weights: tok_emb, final_norm_w, lm_head, layer_tensors required", who);
  if (d->pos_kind == SPEC_POS_LEARNED && !w->d_pos_emb)
    return fail(nullptr, SPEC_ERR_INVALID_ARG, "%s weights: pos_emb required for learned positions", who);
  if (d->norm_kind == SPEC_NORM_LAYER && !w->d_final_norm_b)
    return fail(nullptr, SPEC_ERR_INVALID_ARG, "%s weights: final_norm_b required for LayerNorm", who);
  const bool ln = d->norm_kind == SPEC_NORM_LAYER, hb = d->has_bias != 0, swi = d->ffn_kind == SPEC_FFN_SWIGLU;
  for (int l = 0; l < d->n_layers; ++l) {
    const void *const *T = w->layer_tensors + (size_t)l * SPEC_T_COUNT;
    bool ok = T[SPEC_T_ATTN_NORM_W] && T[SPEC_T_WQ] && T[SPEC_T_WK] && T[SPEC_T_WV] && T[SPEC_T_WO] &&
              T[SPEC_T_FFN_NORM_W] && T[SPEC_T_W1] && T[SPEC_T_W2];
    if (ln) ok = ok && T[SPEC_T_ATTN_NORM_B] && T[SPEC_T_FFN_NORM_B];
    if (hb) ok = ok && T[SPEC_T_BQ] && T[SPEC_T_BK] && T[SPEC_T_BV] && T[SPEC_T_BO];
    if (swi) ok = ok && T[SPEC_T_W3];
    if (hb && !swi) ok = ok && T[SPEC_T_B1] && T[SPEC_T_B2];
    if (!ok) return fail(nullptr, SPEC_ERR_INVALID_ARG, "%s weights: layer %d misses a required tensor", who, l);
  }
  return SPEC_OK;
}

static void *carve(char *&p, size_t bytes) {
  void *r = p;
  p += al256(bytes);
  return r;
}

static int setup_model(spec_ctx *c, Model &m, const spec_model_desc *d, const spec_weights *w, char *&p,
                       size_t w_bytes, size_t kv_area, size_t kv_bytes, int L_pad) {
  m.present = true;
  m.desc = *d;
  m.hd = d->d_model / d->n_heads;
  m.L_pad = L_pad;
  m.fast = fast_supported(*d, c->run.dtype);
  m.layers.resize(d->n_layers);
  void *cursor = p;
  if (m.fast) {
    if (!fast_setup_model(c, m, w, cursor, c->stream)) return fail(c, SPEC_ERR_HIP, "spec_init: weight packing failed");
  } else {
    generic_repack_top(c, m, w, cursor, c->stream);
    for (int l = 0; l < d->n_layers; ++l) generic_repack_layer(c, m, l, w, cursor, c->stream);
  }
  if ((size_t)((char *)cursor - p) > w_bytes) return fail(c, SPEC_ERR_WORKSPACE, "internal: packed weights overflow");
  p += w_bytes;
  m.kv_area_elems = kv_area;
  m.kcache = p;
  m.vcache = p + kv_bytes / 2;
  // stale cache rows are read (and multiplied by exact zeros) by the attention kernel: keep them finite
  generic_zero(p, kv_bytes, c->stream);
  p += kv_bytes;
  return SPEC_OK;
}

extern "C" int spec_init(const spec_model_desc *tgt, const spec_weights *tgt_w, const spec_model_desc *drf,
                         const spec_weights *drf_w, const spec_run_desc *run, void *d_workspace,
                         size_t workspace_bytes, void *hip_stream, spec_ctx **out) {
  if (!out) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_init: out is null");
  *out = nullptr;
  if (!tgt || !tgt_w || !run) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_init: target model, weights and run are required");
  if ((drf == nullptr) != (drf_w == nullptr))
    return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_init: give both the draft description and its weights, or neither");
  size_t need = 0;
  int rc = spec_workspace_bytes(tgt, drf, run, &need);
  if (rc) return rc;
  if ((rc = check_weights(tgt, tgt_w, "target"))) return rc;
  if (drf && (rc = check_weights(drf, drf_w, "draft"))) return rc;
  if (!drf && run->proposal_mode == SPEC_PROPOSALS_DRAFT && run->s_max > 0)
    return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_init: s_max > 0 with SPEC_PROPOSALS_DRAFT needs a draft model");
  if (!d_workspace) return fail(nullptr, SPEC_ERR_WORKSPACE, "spec_init: workspace is null");
  if ((uintptr_t)d_workspace % 256 != 0) return fail(nullptr, SPEC_ERR_WORKSPACE, "spec_init: workspace must be 256-byte aligned");
  if (workspace_bytes < need)
    return fail(nullptr, SPEC_ERR_WORKSPACE, "spec_init: workspace has %zu bytes, %zu needed", workspace_bytes, need);
  // generic attention keeps one fp32 score per key in LDS
  if ((size_t)run->L_max * 4 + 64 > 64 * 1024)
    return fail(nullptr, SPEC_ERR_UNSUPPORTED, "spec_init: L_max above 16368 is not supported");

  spec_ctx *c = new (std::nothrow) spec_ctx();
  if (!c) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_init: out of host memory");
  c->run = *run;
  c->eos = run->eos_id;
  c->stream = (hipStream_t)hip_stream;
  {  // per device: the CU count the launch shapes are chosen for, and the kernels' LDS allowances
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
      c->n_cu = prop.multiProcessorCount;
    gemm_tile_prepare();
    attention_prepare();
  }
  Sizes z = compute_sizes(tgt, drf, run);
  c->M_max = z.M_max;
  char *p = (char *)d_workspace;
  const size_t B = run->B_max, L = run->L_max, s = run->s_max, M = z.M_max, e = dtype_bytes(run->dtype);
  State &S = c->st;
  S.seq = (int32_t *)carve(p, B * L * 4);
  S.n = (int32_t *)carve(p, B * 4);
  S.P_b = (int32_t *)carve(p, B * 4);
  S.gen_cap = (int32_t *)carve(p, B * 4);
  S.l_last = (int32_t *)carve(p, B * 4);
  S.draft_arg = (int32_t *)carve(p, B * 4);
  c->drf.kv_len = (int32_t *)carve(p, B * 4);
  S.t = (int32_t *)carve(p, B * std::max<size_t>(s, 1) * 4);
  S.a = (int32_t *)carve(p, B * (s + 1) * 4);
  S.hist = (unsigned long long *)carve(p, (s + 1) * 8);
  S.counters = (unsigned long long *)carve(p, 16);
  S.sat = (unsigned int *)carve(p, 4);
  size_t d = tgt->d_model, f = tgt->d_ffn, V = tgt->vocab;
  size_t wide = std::max(3 * d, (tgt->ffn_kind == SPEC_FFN_SWIGLU ? 2 : 1) * f);
  if (drf) {
    d = std::max<size_t>(d, drf->d_model);
    f = std::max<size_t>(f, drf->d_ffn);
    V = std::max<size_t>(V, drf->vocab);
    wide = std::max(wide, std::max<size_t>(3 * (size_t)drf->d_model,
                                           (drf->ffn_kind == SPEC_FFN_SWIGLU ? 2 : 1) * (size_t)drf->d_ffn));
  }
  Workspace &W = c->ws;
  W.h = (float *)carve(p, M * d * 4);
  const size_t Mp = (M + 15) / 16 * 16;
  W.x = carve(p, Mp * d * e);
  W.q = carve(p, Mp * d * 4);  // fp32 on the matrix-core path, the model dtype on the generic one
  W.attn = carve(p, Mp * d * e);
  W.act = carve(p, Mp * f * e);
  W.y32 = (float *)carve(p, M * wide * 4);
  W.logits = (float *)carve(p, M * V * 4);
  W.row_tok = (int32_t *)carve(p, M * 4);
  W.row_pos = (int32_t *)carve(p, M * 4);
  W.row_seq = (int32_t *)carve(p, M * 4);
  {
    const size_t NC = (size_t)attn_chunk_of((int)std::max<size_t>(L, 1) - 1) + 1, NTh = (V + 15) / 16;
    c->NC_max = (int)NC;
    W.attn_part = (float *)carve(p, M * d * NC * 4);
    W.attn_ml = (float *)carve(p, M * (d / 64 + 1) * NC * 2 * 4);
    W.head_part = (float *)carve(p, M * NTh * 4);
    W.head_part_idx = (int32_t *)carve(p, M * NTh * 4);
    W.gemm_part = M > 32 ? (float *)carve(p, 8 * Mp * d * 4) : nullptr;
    W.row_inv = (float *)carve(p, M * 4);
    W.row_mean = (float *)carve(p, M * 4);
  }

  rc = setup_model(c, c->tgt, tgt, tgt_w, p, z.tgt_w, z.kv_area_tgt, z.tgt_kv, z.L_pad);
  if (!rc && drf) {
    int32_t *kvlen = c->drf.kv_len;
    rc = setup_model(c, c->drf, drf, drf_w, p, z.drf_w, z.kv_area_drf, z.drf_kv, z.L_pad);
    c->drf.kv_len = kvlen;
  }
  if (!drf) c->drf.kv_len = nullptr;
  if (!rc && (size_t)(p - (char *)d_workspace) > workspace_bytes) rc = fail(c, SPEC_ERR_WORKSPACE, "internal: workspace overflow");
  if (rc) { g_err = c->err; delete c; return rc; }
  // state that kernels read before the first reset writes it
  generic_zero(S.seq, (size_t)((char *)W.h - (char *)S.seq), c->stream);
  hipError_t e1 = hipEventCreate(&c->ev0), e2 = hipEventCreate(&c->ev1);
  hipError_t e3 = hipStreamSynchronize(c->stream);
  hipError_t e4 = hipGetLastError();
  if (e1 != hipSuccess || e2 != hipSuccess || e3 != hipSuccess || e4 != hipSuccess) {
    hipError_t bad = e1 != hipSuccess ? e1 : e2 != hipSuccess ? e2 : e3 != hipSuccess ? e3 : e4;
    rc = fail(nullptr, SPEC_ERR_HIP, "spec_init: %s", hipGetErrorString(bad));
    delete c;
    return rc;
  }
  *out = c;
  return SPEC_OK;
}

extern "C" int spec_set_hidden_dump(spec_ctx *c, float *d_hidden) {
  if (!c) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_set_hidden_dump: ctx is null");
  c->hidden_dump = d_hidden;
  return SPEC_OK;
}

extern "C" int spec_set_sampling(spec_ctx *c, float temperature, const float *d_uniforms, float *d_target_logits,
                                 float *d_draft_logits) {
  if (!c) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_set_sampling: ctx is null");
  if (c->draft_j != 0 || c->verified_s >= 0) return fail(c, SPEC_ERR_STATE, "spec_set_sampling: a round is in progress");
  if (!d_uniforms) {  // back to the greedy rule
    c->smp_u = nullptr; c->smp_tl = c->smp_dl = nullptr; c->smp_T = 0.f;
    return SPEC_OK;
  }
  if (!(temperature > 0.f)) return fail(c, SPEC_ERR_INVALID_ARG, "spec_set_sampling: temperature must be positive");
  if (!d_target_logits) return fail(c, SPEC_ERR_INVALID_ARG, "spec_set_sampling: a buffer for the target's logits is needed");
  if (c->run.proposal_mode == SPEC_PROPOSALS_DRAFT && !d_draft_logits)
    return fail(c, SPEC_ERR_INVALID_ARG, "spec_set_sampling: proposals drawn by the draft model need a buffer for its logits");
  c->smp_T = temperature; c->smp_u = d_uniforms; c->smp_tl = d_target_logits;
  c->smp_dl = c->run.proposal_mode == SPEC_PROPOSALS_DRAFT ? d_draft_logits : nullptr;
  return SPEC_OK;
}

extern "C" int spec_set_draft_logits(spec_ctx *c, float *d_logits) {
  if (!c) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_set_draft_logits: ctx is null");
  if (!c->drf.present) return fail(c, SPEC_ERR_STATE, "spec_set_draft_logits: no draft model");
  c->draft_logits = d_logits;
  return SPEC_OK;
}

extern "C" int spec_read_saturation(spec_ctx *c, int64_t *h_count) {
  if (!c || !h_count) return fail(c, SPEC_ERR_INVALID_ARG, "spec_read_saturation: null argument");
  HIPCHK(c, hipStreamSynchronize(c->stream));
  unsigned int n = 0;
  HIPCHK(c, hipMemcpy(&n, c->st.sat, sizeof n, hipMemcpyDeviceToHost));
  *h_count = (int64_t)n;
  return SPEC_OK;
}

extern "C" int spec_read_proposals(spec_ctx *c, int32_t *h_t) {
  if (!c || !h_t) return fail(c, SPEC_ERR_INVALID_ARG, "spec_read_proposals: null argument");
  if (!c->active) return fail(c, SPEC_ERR_STATE, "spec_read_proposals: no batch; call spec_reset first");
  if (c->run.s_max == 0) return SPEC_OK;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(h_t, c->st.t, (size_t)c->B * c->run.s_max * 4, hipMemcpyDeviceToHost));
  return SPEC_OK;
}

// Per-sequence cap on the speculation length (beyond the paper, whose rounds use one s for the batch).
extern "C" int spec_set_seq_s(spec_ctx *c, const int32_t *d_s_or_null) {
  if (!c) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_set_seq_s: ctx is null");
  if (c->draft_j != 0 || c->verified_s >= 0)
    return fail(c, SPEC_ERR_STATE, "spec_set_seq_s: a round is in progress; finish it with spec_accept_commit first");
  c->seq_s = d_s_or_null;
  return SPEC_OK;
}

// End-of-sequence token (beyond the paper, whose sequences all run to a fixed length).
extern "C" int spec_set_eos(spec_ctx *c, int32_t eos_token) {
  if (!c) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_set_eos: ctx is null");
  if (eos_token < -1 || eos_token >= c->tgt.desc.vocab)
    return fail(c, SPEC_ERR_INVALID_ARG, "spec_set_eos: token %d outside -1..vocab-1=%d", eos_token, c->tgt.desc.vocab - 1);
  if (c->draft_j != 0 || c->verified_s >= 0)
    return fail(c, SPEC_ERR_STATE, "spec_set_eos: a round is in progress; finish it with spec_accept_commit first");
  c->eos = eos_token;
  return SPEC_OK;
}

extern "C" int spec_set_gemm_tuning(spec_ctx *c, int32_t tile_mtw, int32_t tile_nbw, int32_t flags) {
  if (!c) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_set_gemm_tuning: ctx is null");
  const bool tile_auto = tile_mtw == 0 && tile_nbw == 0;
  if (!tile_auto && (tile_mtw < 1 || tile_mtw > 4 || tile_nbw < 2 || tile_nbw > 4))
    return fail(c, SPEC_ERR_INVALID_ARG, "spec_set_gemm_tuning: wave tile must be 0,0 (automatic) or 1..4 x 2..4");
  if (flags < 0 || flags > 3) return fail(c, SPEC_ERR_INVALID_ARG, "spec_set_gemm_tuning: unknown flag bits");
  int t = tile_auto ? 0 : (tile_mtw | (tile_nbw << TUNE_TILE_NBW_SHIFT));
  if (flags & 1) t |= TUNE_ROWRES_OFF;
  if (flags & 2) t |= TUNE_ROWRES_ALWAYS;
  c->gemm_tune = t;
  return SPEC_OK;
}

extern "C" int spec_set_attention_shape(spec_ctx *c, int32_t shape) {
  if (!c) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_set_attention_shape: ctx is null");
  if (shape < 0 || shape > 3) return fail(c, SPEC_ERR_INVALID_ARG, "spec_set_attention_shape: shape must be 0, 1, 2 or 3");
  c->attn_shape = shape;
  return SPEC_OK;
}

extern "C" int spec_kernel_timing(spec_ctx *c, int32_t enable) {
  if (!c) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_kernel_timing: ctx is null");
  c->kt_on = enable != 0;
  return SPEC_OK;
}

extern "C" int spec_read_kernel_timing(spec_ctx *c, int64_t *h_count, double *h_ms) {
  if (!c || !h_count || !h_ms) return fail(c, SPEC_ERR_INVALID_ARG, "spec_read_kernel_timing: null argument");
  HIPCHK(c, hipStreamSynchronize(c->stream));
  for (int i = 0; i < SPEC_KCLASS_COUNT; ++i) { h_count[i] = 0; h_ms[i] = 0.0; }
  for (size_t i = 0; i < c->kt_used; ++i) {
    float ms = 0.f;
    HIPCHK(c, hipEventElapsedTime(&ms, c->kt_ev[2 * i], c->kt_ev[2 * i + 1]));
    const int cls = c->kt_cls[i];
    if (cls >= 0 && cls < SPEC_KCLASS_COUNT) { h_count[cls] += 1; h_ms[cls] += ms; }
  }
  c->kt_used = 0;
  return SPEC_OK;
}

extern "C" int spec_destroy(spec_ctx *c) {
  if (!c) return SPEC_OK;
  for (hipEvent_t e : c->kt_ev) (void)hipEventDestroy(e);
  if (c->ev0) (void)hipEventDestroy(c->ev0);
  if (c->ev1) (void)hipEventDestroy(c->ev1);
  delete c;
  return SPEC_OK;
}

// ------------------------------------------------------------------ forward pass
enum HeadMode { HEAD_NONE = 0, HEAD_ALL = 1, HEAD_LAST = 2 };

// One forward pass of a model over B*q rows: embed -> layers -> (final norm, LM head,
// arg-max for the rows that need a token).
static int forward_pass(spec_ctx *c, Model &m, const PassArgs &pa, HeadMode head, float *logits_out,
                        int32_t *arg_out, int arg_stride, int max_pos) {
  const int M = pa.B * pa.q;
  hipStream_t st = c->stream;
  max_pos = std::max(0, std::min(max_pos, c->run.L_max - 1));
  KScope whole(c, &m == &c->drf ? SPEC_KCLASS_DRAFT_PASS : -1);
  { KScope k(c, &m == &c->tgt ? SPEC_KCLASS_OTHER : -1); launch_assemble_embed(c, m, pa, st); }
  float *dump = (&m == &c->tgt) ? c->hidden_dump : nullptr;
  const size_t hbytes = (size_t)M * m.desc.d_model * sizeof(float);
  if (dump) generic_copy(c->ws.h, dump, hbytes, st);
  c->x_ssq = false;  // the rows in ws.x come from the embedding
  for (int l = 0; l < m.desc.n_layers; ++l) {
    if (m.fast) fast_layer(c, m, l, pa.B, pa.q, pa.b0, pa.seq_groups, max_pos, st);
    else generic_layer(c, m, l, M, pa.q, pa.b0, pa.seq_groups, st);
    if (dump) generic_copy(c->ws.h, (char *)dump + (size_t)(l + 1) * hbytes, hbytes, st);
  }
  if (head != HEAD_NONE) {
    const bool last = head == HEAD_LAST;
    const int Mh = last ? pa.B : M;
    const int last_of_q = last ? pa.q : 0;  // the final norm gathers the rows that need a token
    if (m.fast) {
      fast_head(c, m, Mh, last_of_q, logits_out, last ? 1 : pa.q, arg_stride, arg_out, st);
    } else {
      float *lg = logits_out ? logits_out : c->ws.logits;
      generic_head(c, m, Mh, last_of_q, lg, st);
      launch_argmax_rows(lg, Mh, m.desc.vocab, last ? 1 : pa.q, arg_stride, arg_out, st);
    }
  }
  HIPCHK(c, hipGetLastError());
  return SPEC_OK;
}

// ------------------------------------------------------------------ prefill
// The first P-1 prompt tokens of the sequences at slots b0 .. b0+B-1 through both models, in passes of up to
// M_max rows.  A sequence's share of a pass is cut into groups of Q_LIMIT rows (the attention query tile) at
// consecutive positions; all groups of a sequence read and write that sequence's cache, so few sequences with
// long prompts need few passes over the weights (one sequence, M_max >= P-1: a single pass).
static int prefill(spec_ctx *c, int b0, int B, int P) {
  int per = std::max(1, c->M_max / B);
  // The tiled GEMMs' time grows in steps of 128 rows (a pass of 576 rows costs what 640 would): the largest row count
  // that is a whole number of such steps, if it is within a quarter of the largest that fits, costs least per row
  // (64 sequences: 8 positions per pass, 512 rows, instead of 9: 7B shape 204 -> 169 ms for 8128 prompt tokens).
  for (int p = per; p >= 1 && 4 * p >= 3 * per; --p)
    if ((B * p) % 128 == 0) { per = p; break; }
  // Fewer positions per sequence than the attention's query tile holds (16) leave the tiles half empty, and every pass
  // reads the cached prefix again: then take fewer sequences per pass and a full tile of each, where the batch
  // divides evenly (32 sequences x 2047 prompt tokens of the 33B shape: 16 x 16 rows per pass instead of 32 x 8).
  int Bs = B;
  if (per < Q_LIMIT && P - 1 > per) {
    const int fewer = B * per / Q_LIMIT;
    if (fewer >= 1 && B % fewer == 0) { Bs = fewer; per = Q_LIMIT; }
  }
  const int q = std::min(Q_LIMIT, per), g = std::max(1, per / q);
  for (int bs = 0; bs < B; bs += Bs)
    for (int base = 0; base < P - 1; base += g * q) {
      const int left = P - 1 - base;
      const int gp = std::min(g, (left + q - 1) / q);          // groups per sequence that still hold positions
      PassArgs pa{PASS_PREFILL, Bs * gp, q, base, P, c->run.s_max, c->run.L_max, b0 + bs, gp};
      const int max_pos = base + std::min(left, gp * q) - 1;
      int rc = forward_pass(c, c->tgt, pa, HEAD_NONE, nullptr, nullptr, 0, max_pos);
      if (!rc && c->drf.present) rc = forward_pass(c, c->drf, pa, HEAD_NONE, nullptr, nullptr, 0, max_pos);
      if (rc) return rc;
    }
  return SPEC_OK;
}

// ------------------------------------------------------------------ reset
// h_len: null (every sequence P tokens long) or B prompt lengths in 1..P, P then being the row stride of d_prompt
static int do_reset(spec_ctx *c, int32_t B, const int32_t *d_prompt, int32_t P, const int32_t *h_len, bool prefill,
                    const char *who) {
  if (!c) return fail(nullptr, SPEC_ERR_INVALID_ARG, "%s: ctx is null", who);
  if (!d_prompt) return fail(c, SPEC_ERR_INVALID_ARG, "%s: prompt is null", who);
  if (B < 1 || B > c->run.B_max) return fail(c, SPEC_ERR_CAPACITY, "%s: B=%d outside 1..B_max=%d", who, B, c->run.B_max);
  if (P < 1) return fail(c, SPEC_ERR_INVALID_ARG, "%s: P must be at least 1", who);
  const int32_t stride = P;
  if (h_len) {  // the longest prompt decides what has to fit
    int32_t longest = 0;
    for (int b = 0; b < B; ++b) {
      if (h_len[b] < 1 || h_len[b] > stride)
        return fail(c, SPEC_ERR_INVALID_ARG, "%s: length %d of sequence %d outside 1..%d", who, h_len[b], b, stride);
      longest = std::max(longest, h_len[b]);
    }
    P = longest;
  }
  if ((long long)P + c->run.gen_max + c->run.s_max > c->run.L_max)
    return fail(c, SPEC_ERR_CAPACITY, "%s: P + gen_max + s_max = %lld exceeds L_max = %d", who,
                (long long)P + c->run.gen_max + c->run.s_max, c->run.L_max);
  for (Model *m : {&c->tgt, &c->drf})
    if (m->present && m->desc.pos_kind == SPEC_POS_LEARNED && P + c->run.gen_max + c->run.s_max > m->desc.max_pos)
      return fail(c, SPEC_ERR_CAPACITY, "%s: positions would exceed the learned position table (max_pos=%d)", who,
                  m->desc.max_pos);
  c->B = B;
  c->P = P;
  if (h_len) c->P_host.assign(h_len, h_len + B);
  else c->P_host.assign((size_t)B, P);
  c->n_ub = P;
  c->active = true;
  c->draft_j = 0;
  c->draft_lag = 1;
  c->verified_s = -1;
  c->proposals_ready = false;
  if (h_len) {  // in stream order, and done with the host buffer before anything can change it
    HIPCHK(c, hipMemcpyAsync(c->st.P_b, c->P_host.data(), (size_t)B * 4, hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
  }
  launch_state_reset(c, d_prompt, stride, h_len != nullptr, c->stream);
  if (prefill) {
    int rc = ::prefill(c, 0, B, P);
    if (rc) return rc;
  }
  HIPCHK(c, hipGetLastError());
  return SPEC_OK;
}

extern "C" int spec_reset(spec_ctx *c, int32_t B, const int32_t *d_prompt, int32_t P) {
  return do_reset(c, B, d_prompt, P, nullptr, true, "spec_reset");
}
extern "C" int spec_reset_ragged(spec_ctx *c, int32_t B, const int32_t *d_prompt, int32_t P_stride, const int32_t *h_len) {
  if (c && !h_len) return fail(c, SPEC_ERR_INVALID_ARG, "spec_reset_ragged: lengths are null");
  return do_reset(c, B, d_prompt, P_stride, h_len, true, "spec_reset_ragged");
}
extern "C" int spec_reset_noprefill(spec_ctx *c, int32_t B, const int32_t *d_prompt, int32_t P) {
  return do_reset(c, B, d_prompt, P, nullptr, false, "spec_reset_noprefill");
}

// Continuous batching: one slot of the running batch starts over with a new prompt (of any length that fits);
// the other sequences keep their state.  The slot's prompt runs through both models in a pass of its own
// (B = 1 at batch slot b), so its cost is that of a single-sequence prefill.
extern "C" int spec_admit(spec_ctx *c, int32_t b, const int32_t *d_prompt, int32_t P) {
  if (!c) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_admit: ctx is null");
  if (!c->active) return fail(c, SPEC_ERR_STATE, "spec_admit: no batch; call spec_reset first");
  if (!d_prompt) return fail(c, SPEC_ERR_INVALID_ARG, "spec_admit: prompt is null");
  if (b < 0 || b >= c->B) return fail(c, SPEC_ERR_INVALID_ARG, "spec_admit: slot %d outside 0..B-1=%d", b, c->B - 1);
  if (P < 1) return fail(c, SPEC_ERR_INVALID_ARG, "spec_admit: P must be at least 1");
  if ((long long)P + c->run.gen_max + c->run.s_max > c->run.L_max)
    return fail(c, SPEC_ERR_CAPACITY, "spec_admit: P + gen_max + s_max = %lld exceeds L_max = %d",
                (long long)P + c->run.gen_max + c->run.s_max, c->run.L_max);
  for (Model *m : {&c->tgt, &c->drf})
    if (m->present && m->desc.pos_kind == SPEC_POS_LEARNED && P + c->run.gen_max + c->run.s_max > m->desc.max_pos)
      return fail(c, SPEC_ERR_CAPACITY, "spec_admit: positions would exceed the learned position table (max_pos=%d)",
                  m->desc.max_pos);
  if (c->draft_j != 0 || c->verified_s >= 0)
    return fail(c, SPEC_ERR_STATE, "spec_admit: a round is in progress; finish it with spec_accept_commit first");
  launch_state_admit(c, b, d_prompt, P, c->stream);
  c->P_host[(size_t)b] = P;
  c->n_ub = std::max(c->n_ub, (int)P);
  int rc = prefill(c, b, 1, P);
  if (rc) return rc;
  HIPCHK(c, hipGetLastError());
  return SPEC_OK;
}

extern "C" int spec_rewind(spec_ctx *c) {
  if (!c) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_rewind: ctx is null");
  if (!c->active) return fail(c, SPEC_ERR_STATE, "spec_rewind: no batch; call spec_reset first");
  c->draft_j = 0;
  c->draft_lag = 1;
  c->verified_s = -1;
  c->proposals_ready = false;
  c->n_ub = *std::max_element(c->P_host.begin(), c->P_host.end());
  launch_state_reset(c, nullptr, 1, false, c->stream);
  HIPCHK(c, hipGetLastError());
  return SPEC_OK;
}

// ------------------------------------------------------------------ proposals
extern "C" int spec_set_proposal_table(spec_ctx *c, const int32_t *d_table) {
  if (!c) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_set_proposal_table: ctx is null");
  if (c->run.proposal_mode != SPEC_PROPOSALS_EXTERNAL)
    return fail(c, SPEC_ERR_STATE, "spec_set_proposal_table: context was created with SPEC_PROPOSALS_DRAFT");
  c->prop_table = d_table;  // NULL clears it
  return SPEC_OK;
}

extern "C" int spec_set_proposals(spec_ctx *c, const int32_t *d_tok, int32_t s) {
  if (!c) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_set_proposals: ctx is null");
  if (c->run.proposal_mode != SPEC_PROPOSALS_EXTERNAL)
    return fail(c, SPEC_ERR_STATE, "spec_set_proposals: context was created with SPEC_PROPOSALS_DRAFT");
  if (!c->active) return fail(c, SPEC_ERR_STATE, "spec_set_proposals: no batch; call spec_reset first");
  if (s < 0 || s > c->run.s_max) return fail(c, SPEC_ERR_CAPACITY, "spec_set_proposals: s=%d outside 0..s_max=%d", s, c->run.s_max);
  if (s > 0 && !d_tok) return fail(c, SPEC_ERR_INVALID_ARG, "spec_set_proposals: tokens are null");
  if (c->draft_j != 0 || c->verified_s >= 0)
    return fail(c, SPEC_ERR_STATE, "spec_set_proposals: call it before the round's first draft step");
  launch_copy_proposals(c, d_tok, s, c->stream);
  c->proposals_ready = true;
  HIPCHK(c, hipGetLastError());
  return SPEC_OK;
}

// proposals for the coming round from the table, if that is how they are supplied
static int ensure_proposals(spec_ctx *c, int s, const char *who) {
  if (c->run.proposal_mode != SPEC_PROPOSALS_EXTERNAL || s == 0 || c->proposals_ready) return SPEC_OK;
  if (!c->prop_table)
    return fail(c, SPEC_ERR_STATE, "%s: external proposals expected; call spec_set_proposals or spec_set_proposal_table", who);
  launch_fill_proposals(c, s, c->stream);
  c->proposals_ready = true;
  return SPEC_OK;
}

// ------------------------------------------------------------------ draft step
extern "C" int spec_draft_step(spec_ctx *c, int32_t j) {
  if (!c) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_draft_step: ctx is null");
  if (!c->active) return fail(c, SPEC_ERR_STATE, "spec_draft_step: no batch; call spec_reset first");
  if (!c->drf.present) return fail(c, SPEC_ERR_STATE, "spec_draft_step: no draft model");
  if (c->verified_s >= 0) return fail(c, SPEC_ERR_STATE, "spec_draft_step: a verify step is waiting for spec_accept_commit");
  if (j < 1 || j > c->run.s_max) return fail(c, SPEC_ERR_CAPACITY, "spec_draft_step: j=%d outside 1..s_max=%d", j, c->run.s_max);
  if (j != c->draft_j + 1) return fail(c, SPEC_ERR_STATE, "spec_draft_step: step %d expected, got %d", c->draft_j + 1, j);
  const bool ext = c->run.proposal_mode == SPEC_PROPOSALS_EXTERNAL;
  if (ext && j >= 2 && !c->proposals_ready)
    return fail(c, SPEC_ERR_STATE, "spec_draft_step: external proposals must be set before draft step 2");
  int rc;
  // the draft's greedy token is t_j: the arg-max kernel writes it straight into the proposals (row stride s_max);
  // with external proposals it goes to a scratch word per sequence instead
  int32_t *arg_out = ext ? c->st.draft_arg : c->st.t + (j - 1);
  const int arg_stride = ext ? 1 : c->run.s_max;
  float *lg = c->draft_logits;
  // sampling: the step's logits are kept for the verification, and t_j is drawn from them instead of their arg-max
  const bool draw = c->smp_u && !ext;
  if (draw) {
    lg = c->smp_dl + (size_t)(j - 1) * c->run.B_max * c->drf.desc.vocab;
    arg_out = c->st.draft_arg;
  }
  const int arg_stride_used = draw ? 1 : arg_stride;
  if (j == 1) {
    if (ext && c->prop_table && !c->proposals_ready) {
      // later draft steps ingest t_1.. : fetch them now (all s_max; verify uses the first s)
      launch_fill_proposals(c, c->run.s_max, c->stream);
      c->proposals_ready = true;
    }
    // The draft's cache is at most draft_lag tokens behind the committed sequences (2 after a round with draft
    // steps, one more per round without).  A pass takes q_cap positions per sequence: what lies further back is
    // ingested by passes without a head first, the last pass ends at position n_b - 1 and yields t_1.
    const int q_cap = std::max(1, std::min(Q_LIMIT, c->M_max / c->B));
    int lag = std::max(1, std::min(c->draft_lag, c->n_ub));
    rc = SPEC_OK;
    while (lag > q_cap && !rc) {
      PassArgs pa{PASS_DRAFT_FIRST, c->B, q_cap, lag - q_cap, c->P, c->run.s_max, c->run.L_max};
      rc = forward_pass(c, c->drf, pa, HEAD_NONE, nullptr, nullptr, 0, c->n_ub - 1);
      lag -= q_cap;
    }
    if (!rc) {
      PassArgs pa{PASS_DRAFT_FIRST, c->B, lag, 0, c->P, c->run.s_max, c->run.L_max};
      rc = forward_pass(c, c->drf, pa, HEAD_LAST, lg, arg_out, arg_stride_used, c->n_ub - 1);
    }
  } else {
    PassArgs pa{PASS_DRAFT_NEXT, c->B, 1, j, c->P, c->run.s_max, c->run.L_max};
    rc = forward_pass(c, c->drf, pa, HEAD_LAST, lg, arg_out, arg_stride_used, c->n_ub + j - 2);
  }
  if (rc) return rc;
  if (draw) {  // t_j decides the token at position n_b + j - 1
    const int V = c->drf.desc.vocab;
    launch_sample_rows(lg, c->B, V, c->smp_T, c->smp_u, c->st.n, j - 1, c->run.L_max, c->st.t + (j - 1), c->run.s_max, c->stream);
    if (c->draft_logits) generic_copy(lg, c->draft_logits, (size_t)c->B * V * sizeof(float), c->stream);
  }
  c->draft_j = j;
  HIPCHK(c, hipGetLastError());
  return SPEC_OK;
}

// ------------------------------------------------------------------ verify
extern "C" int spec_verify_step(spec_ctx *c, int32_t s, float *d_logits_or_null) {
  if (!c) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_verify_step: ctx is null");
  if (!c->active) return fail(c, SPEC_ERR_STATE, "spec_verify_step: no batch; call spec_reset first");
  if (s < 0 || s > c->run.s_max) return fail(c, SPEC_ERR_CAPACITY, "spec_verify_step: s=%d outside 0..s_max=%d", s, c->run.s_max);
  if (c->verified_s >= 0) return fail(c, SPEC_ERR_STATE, "spec_verify_step: previous verify step not committed yet");
  if (c->run.proposal_mode == SPEC_PROPOSALS_DRAFT && c->draft_j != s)
    return fail(c, SPEC_ERR_STATE, "spec_verify_step: s=%d needs %d draft steps first, %d were run", s, s, c->draft_j);
  if (c->draft_j != 0 && c->draft_j != s)
    return fail(c, SPEC_ERR_STATE, "spec_verify_step: %d draft steps were run for s=%d", c->draft_j, s);
  int rc = ensure_proposals(c, s, "spec_verify_step");
  if (rc) return rc;
  PassArgs pa{PASS_VERIFY, c->B, s + 1, 0, c->P, c->run.s_max, c->run.L_max};
  float *lg = d_logits_or_null ? d_logits_or_null : c->smp_u ? c->smp_tl : nullptr;
  rc = forward_pass(c, c->tgt, pa, HEAD_ALL, lg, c->st.a, c->run.s_max + 1, c->n_ub - 1 + s);
  if (rc) return rc;
  if (c->smp_u) {  // the sampling rule in place of the arg-max: row j decides the token at position n_b + j
    KScope k(c, SPEC_KCLASS_OTHER);
    launch_sample_verify(lg, c->smp_dl, c->run.B_max, c->B, s, c->tgt.desc.vocab, c->smp_T, c->st.t, c->run.s_max, c->seq_s,
                         c->smp_u, c->st.n, c->run.L_max, c->st.a, c->run.s_max + 1, c->stream);
    HIPCHK(c, hipGetLastError());
  }
  c->verified_s = s;
  return SPEC_OK;
}

// ------------------------------------------------------------------ accept / commit
extern "C" int spec_accept_commit(spec_ctx *c, int32_t s) {
  if (!c) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_accept_commit: ctx is null");
  if (!c->active) return fail(c, SPEC_ERR_STATE, "spec_accept_commit: no batch; call spec_reset first");
  if (c->verified_s < 0) return fail(c, SPEC_ERR_STATE, "spec_accept_commit: no verify step to commit");
  if (s != c->verified_s) return fail(c, SPEC_ERR_STATE, "spec_accept_commit: verify step ran with s=%d, got s=%d", c->verified_s, s);
  { KScope k(c, SPEC_KCLASS_OTHER); launch_accept(c, s, c->stream); }
  c->n_ub = std::min(c->n_ub + s + 1, *std::max_element(c->P_host.begin(), c->P_host.end()) + c->run.gen_max);
  if (c->drf.present) c->draft_lag = c->draft_j > 0 ? 2 : std::min(c->draft_lag + 1, c->n_ub);
  c->draft_j = 0;
  c->verified_s = -1;
  c->proposals_ready = false;
  HIPCHK(c, hipGetLastError());
  return SPEC_OK;
}

extern "C" int spec_round(spec_ctx *c, int32_t s, int32_t n_rounds) {
  if (!c) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_round: ctx is null");
  if (!c->active) return fail(c, SPEC_ERR_STATE, "spec_round: no batch; call spec_reset first");
  if (s < 0 || s > c->run.s_max) return fail(c, SPEC_ERR_CAPACITY, "spec_round: s=%d outside 0..s_max=%d", s, c->run.s_max);
  if (n_rounds < 0) return fail(c, SPEC_ERR_INVALID_ARG, "spec_round: n_rounds is negative");
  if (c->draft_j != 0 || c->verified_s >= 0) return fail(c, SPEC_ERR_STATE, "spec_round: a round is already in progress");
  const bool ext = c->run.proposal_mode == SPEC_PROPOSALS_EXTERNAL;
  if (ext && s > 0 && !c->prop_table && !(n_rounds == 1 && c->proposals_ready))
    return fail(c, SPEC_ERR_STATE, "spec_round: external proposals need a table (spec_set_proposal_table)");
  if (!ext && s > 0 && !c->drf.present) return fail(c, SPEC_ERR_STATE, "spec_round: no draft model");
  for (int r = 0; r < n_rounds; ++r) {
    int rc = SPEC_OK;
    if (c->drf.present)
      for (int j = 1; j <= s && !rc; ++j) rc = spec_draft_step(c, j);
    if (!rc) rc = spec_verify_step(c, s, nullptr);
    if (!rc) rc = spec_accept_commit(c, s);
    if (rc) return rc;
  }
  return SPEC_OK;
}

// ------------------------------------------------------------------ adaptive policy
static int lut_lookup(const std::vector<int32_t> &Bs, const std::vector<int32_t> &lut, int B) {
  // smaller entry of the two nearest profiled sizes; ends clamp
  const int n = (int)Bs.size();
  if (B <= Bs[0]) return lut[0];
  if (B >= Bs[n - 1]) return lut[n - 1];
  int hi = 0;
  while (Bs[hi] < B) ++hi;
  if (Bs[hi] == B) return lut[hi];
  return std::min(lut[hi - 1], lut[hi]);
}

static int check_batch_list(spec_ctx *c, const int32_t *h_batch_sizes, int32_t n_b, const char *who) {
  if (!h_batch_sizes || n_b < 1) return fail(c, SPEC_ERR_INVALID_ARG, "%s: batch size list is empty", who);
  for (int i = 0; i < n_b; ++i) {
    if (h_batch_sizes[i] < 1) return fail(c, SPEC_ERR_INVALID_ARG, "%s: batch sizes must be positive", who);
    if (i && h_batch_sizes[i] <= h_batch_sizes[i - 1])
      return fail(c, SPEC_ERR_INVALID_ARG, "%s: batch sizes must be strictly ascending", who);
  }
  return SPEC_OK;
}

extern "C" int spec_set_lut(spec_ctx *c, const int32_t *h_batch_sizes, const int32_t *h_lut, int32_t n_b) {
  if (!c) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_set_lut: ctx is null");
  int rc = check_batch_list(c, h_batch_sizes, n_b, "spec_set_lut");
  if (rc) return rc;
  if (!h_lut) return fail(c, SPEC_ERR_INVALID_ARG, "spec_set_lut: lut is null");
  for (int i = 0; i < n_b; ++i)
    if (h_lut[i] < 0 || h_lut[i] > c->run.s_max)
      return fail(c, SPEC_ERR_CAPACITY, "spec_set_lut: entry %d = %d outside 0..s_max=%d", i, h_lut[i], c->run.s_max);
  c->lut_B.assign(h_batch_sizes, h_batch_sizes + n_b);
  c->lut_s.assign(h_lut, h_lut + n_b);
  return SPEC_OK;
}

extern "C" int spec_choose_s(const spec_ctx *c, int32_t B, int32_t *h_s_out) {
  if (!c || !h_s_out) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_choose_s: null argument");
  if (c->lut_B.empty()) return fail(const_cast<spec_ctx *>(c), SPEC_ERR_STATE, "spec_choose_s: no look-up table; profile or call spec_set_lut");
  if (B < 1) return fail(const_cast<spec_ctx *>(c), SPEC_ERR_INVALID_ARG, "spec_choose_s: B must be positive");
  *h_s_out = lut_lookup(c->lut_B, c->lut_s, B);
  return SPEC_OK;
}

extern "C" int spec_profile_and_choose_s(spec_ctx *c, const int32_t *h_batch_sizes, int32_t n_b, int32_t s_max_profile,
                                         const int32_t *d_prompt, int32_t P, int32_t gen, int32_t *h_lut_out,
                                         float *h_grid) {
  if (!c) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_profile_and_choose_s: ctx is null");
  int rc = check_batch_list(c, h_batch_sizes, n_b, "spec_profile_and_choose_s");
  if (rc) return rc;
  if (!h_lut_out || !d_prompt) return fail(c, SPEC_ERR_INVALID_ARG, "spec_profile_and_choose_s: null argument");
  if (h_batch_sizes[n_b - 1] > c->run.B_max)
    return fail(c, SPEC_ERR_CAPACITY, "spec_profile_and_choose_s: batch size %d exceeds B_max=%d", h_batch_sizes[n_b - 1], c->run.B_max);
  if (s_max_profile < 0 || s_max_profile > c->run.s_max)
    return fail(c, SPEC_ERR_CAPACITY, "spec_profile_and_choose_s: s_max_profile=%d outside 0..s_max=%d", s_max_profile, c->run.s_max);
  if (gen < 1 || gen > c->run.gen_max)
    return fail(c, SPEC_ERR_CAPACITY, "spec_profile_and_choose_s: gen=%d outside 1..gen_max=%d", gen, c->run.gen_max);
  const bool ext = c->run.proposal_mode == SPEC_PROPOSALS_EXTERNAL;
  if (ext && s_max_profile > 0 && !c->prop_table)
    return fail(c, SPEC_ERR_STATE, "spec_profile_and_choose_s: external proposals need a table");
  if (!ext && s_max_profile > 0 && !c->drf.present) return fail(c, SPEC_ERR_STATE, "spec_profile_and_choose_s: no draft model");
  const int nS = s_max_profile + 1;
  std::vector<double> grid((size_t)n_b * nS), us_round((size_t)n_b * nS);
  std::vector<double> tok_s(nS, 0.0), seq_rounds_s(nS, 0.0);  // per s, pooled over the batch sizes
  std::vector<int32_t> lut(n_b);
  struct CapsOff {  // the profiling stage times uniform rounds: per-sequence caps and the end token are set aside until it returns
    spec_ctx *c; const int32_t *saved; int32_t saved_eos;
    explicit CapsOff(spec_ctx *ctx) : c(ctx), saved(ctx->seq_s), saved_eos(ctx->eos) { c->seq_s = nullptr; c->eos = -1; }
    ~CapsOff() { c->seq_s = saved; c->eos = saved_eos; }
  } caps_off(c);
  for (int bi = 0; bi < n_b; ++bi) {
    const int B = h_batch_sizes[bi];
    // rows of d_prompt have stride P: the first B rows are the batch
    rc = spec_reset(c, B, d_prompt, P);
    if (rc) return rc;
    for (int s = 0; s < nS; ++s) {
      if ((rc = spec_rewind(c))) return rc;
      // a round emits at most s+1 tokens per sequence: this many rounds cannot finish any sequence,
      // so every round of the timed region does full work
      const int rounds = std::max(1, gen / (s + 1));
      if ((rc = spec_round(c, s, 1))) return rc;  // warm-up round
      if ((rc = spec_rewind(c))) return rc;
      HIPCHK(c, hipEventRecord(c->ev0, c->stream));
      if ((rc = spec_round(c, s, rounds))) return rc;
      HIPCHK(c, hipEventRecord(c->ev1, c->stream));
      HIPCHK(c, hipEventSynchronize(c->ev1));
      float ms = 0.f;
      HIPCHK(c, hipEventElapsedTime(&ms, c->ev0, c->ev1));
      unsigned long long cnt[2] = {0, 0};
      HIPCHK(c, hipMemcpy(cnt, c->st.counters, sizeof cnt, hipMemcpyDeviceToHost));
      us_round[(size_t)bi * nS + s] = (double)ms * 1000.0 / rounds;
      tok_s[s] += (double)cnt[0];
      seq_rounds_s[s] += (double)B * rounds;
    }
  }
  // Time per emitted token per sequence = time of a round / tokens a sequence emits per round.  A round's time is
  // a property of (B, s) and repeats to a fraction of a per cent; the tokens per round depend on s and on how well the
  // proposals agree with the target, not on B (Alg. 1 has no term that couples sequences), and a single small batch
  // sees only a few dozen acceptance draws -- so they are pooled over all batch sizes of the run.
  for (int bi = 0; bi < n_b; ++bi) {
    for (int s = 0; s < nS; ++s) {
      const double per_round = seq_rounds_s[s] > 0 ? tok_s[s] / seq_rounds_s[s] : 0.0;
      grid[(size_t)bi * nS + s] = per_round > 0 ? us_round[(size_t)bi * nS + s] / per_round : 1e30;
    }
    // arg-min over s; within 1 % of the minimum the smaller s wins
    const double *row = &grid[(size_t)bi * nS];
    double best = *std::min_element(row, row + nS);
    int pick = 0;
    while (row[pick] > best * 1.01) ++pick;
    lut[bi] = pick;
  }
  if ((rc = spec_rewind(c))) return rc;
  c->lut_B.assign(h_batch_sizes, h_batch_sizes + n_b);
  c->lut_s = lut;
  std::copy(lut.begin(), lut.end(), h_lut_out);
  if (h_grid) for (size_t i = 0; i < grid.size(); ++i) h_grid[i] = (float)grid[i];
  return SPEC_OK;
}

// ------------------------------------------------------------------ read-back
extern "C" int spec_read_output(spec_ctx *c, int32_t *h_tokens, int32_t *h_len, int64_t *h_hist) {
  if (!c) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_read_output: ctx is null");
  if (!c->active) return fail(c, SPEC_ERR_STATE, "spec_read_output: no batch; call spec_reset first");
  if (!h_tokens || !h_len) return fail(c, SPEC_ERR_INVALID_ARG, "spec_read_output: null argument");
  HIPCHK(c, hipStreamSynchronize(c->stream));
  std::vector<int32_t> n(c->B);
  HIPCHK(c, hipMemcpy(n.data(), c->st.n, (size_t)c->B * 4, hipMemcpyDeviceToHost));
  const int G = c->run.gen_max;
  for (int b = 0; b < c->B; ++b) {
    const int Pb = c->P_host[(size_t)b];
    int len = std::max(0, std::min(n[b] - Pb, G));
    h_len[b] = len;
    if (len)
      HIPCHK(c, hipMemcpy(h_tokens + (size_t)b * G, c->st.seq + (size_t)b * c->run.L_max + Pb, (size_t)len * 4,
                          hipMemcpyDeviceToHost));
  }
  if (h_hist) {
    static_assert(sizeof(unsigned long long) == sizeof(int64_t), "hist width");
    HIPCHK(c, hipMemcpy(h_hist, c->st.hist, (size_t)(c->run.s_max + 1) * 8, hipMemcpyDeviceToHost));
  }
  return SPEC_OK;
}

extern "C" int spec_read_state(spec_ctx *c, int32_t *h_n, int32_t *h_kv_draft, int32_t *h_l_last, int32_t *h_argmax) {
  if (!c) return fail(nullptr, SPEC_ERR_INVALID_ARG, "spec_read_state: ctx is null");
  if (!c->active) return fail(c, SPEC_ERR_STATE, "spec_read_state: no batch; call spec_reset first");
  HIPCHK(c, hipStreamSynchronize(c->stream));
  const size_t B = c->B;
  if (h_n) HIPCHK(c, hipMemcpy(h_n, c->st.n, B * 4, hipMemcpyDeviceToHost));
  if (h_kv_draft) {
    if (c->drf.kv_len) HIPCHK(c, hipMemcpy(h_kv_draft, c->drf.kv_len, B * 4, hipMemcpyDeviceToHost));
    else std::fill(h_kv_draft, h_kv_draft + B, 0);
  }
  if (h_l_last) HIPCHK(c, hipMemcpy(h_l_last, c->st.l_last, B * 4, hipMemcpyDeviceToHost));
  if (h_argmax) HIPCHK(c, hipMemcpy(h_argmax, c->st.a, B * (size_t)(c->run.s_max + 1) * 4, hipMemcpyDeviceToHost));
  return SPEC_OK;
}

// ------------------------------------------------------------------ KV import / export
static int kv_io(spec_ctx *c, int32_t which, int32_t layer, int32_t B, int32_t len, void *k, void *v, bool import_,
                 const char *who) {
  if (!c) return fail(nullptr, SPEC_ERR_INVALID_ARG, "%s: ctx is null", who);
  if (which != SPEC_MODEL_TARGET && which != SPEC_MODEL_DRAFT) return fail(c, SPEC_ERR_INVALID_ARG, "%s: unknown model %d", who, which);
  Model &m = which == SPEC_MODEL_TARGET ? c->tgt : c->drf;
  if (!m.present) return fail(c, SPEC_ERR_STATE, "%s: no draft model", who);
  if (layer < 0 || layer >= m.desc.n_layers) return fail(c, SPEC_ERR_INVALID_ARG, "%s: layer %d outside 0..%d", who, layer, m.desc.n_layers - 1);
  if (B < 1 || B > c->run.B_max) return fail(c, SPEC_ERR_CAPACITY, "%s: B=%d outside 1..B_max=%d", who, B, c->run.B_max);
  if (len < 0 || len > c->run.L_max) return fail(c, SPEC_ERR_CAPACITY, "%s: len=%d outside 0..L_max=%d", who, len, c->run.L_max);
  if (len > 0 && (!k || !v)) return fail(c, SPEC_ERR_INVALID_ARG, "%s: null buffer", who);
  launch_kv_convert(c, m, layer, B, len, k, v, import_, c->stream);
  HIPCHK(c, hipGetLastError());
  return SPEC_OK;
}
extern "C" int spec_kv_import(spec_ctx *c, int32_t which, int32_t layer, int32_t B, int32_t len, const void *d_k,
                              const void *d_v) {
  return kv_io(c, which, layer, B, len, const_cast<void *>(d_k), const_cast<void *>(d_v), true, "spec_kv_import");
}
extern "C" int spec_kv_export(spec_ctx *c, int32_t which, int32_t layer, int32_t B, int32_t len, void *d_k, void *d_v) {
  return kv_io(c, which, layer, B, len, d_k, d_v, false, "spec_kv_export");
}
