// The 16-bit path: model set-up (weight packing) and the per-layer launch sequence built
// from the matrix-core kernels.
#include "spec_internal.h"
#include "mfma_gemm.h"
#include <algorithm>
#include <vector>

namespace spec {

static size_t al256f(size_t b) { return (b + 255) & ~(size_t)255; }

bool fast_supported(const spec_model_desc &D, int dtype) {
  if (dtype != SPEC_DTYPE_BF16 && dtype != SPEC_DTYPE_F16) return false;
  const int hd = D.d_model / D.n_heads;
  if (hd != 64 && hd != 128) return false;
  if (D.d_model % 32 != 0 || D.d_ffn % 32 != 0) return false;
  return true;
}

struct FastDims {
  PackedDims qkv, o, w13, w2, head;
};
static FastDims fast_dims(const spec_model_desc &D) {
  FastDims f;
  const int d = D.d_model, ff = D.d_ffn;
  f.qkv = packed_dims(3 * d, d);
  f.o = packed_dims(d, d);
  f.w13 = packed_dims(D.ffn_kind == SPEC_FFN_SWIGLU ? 2 * ff : ff, d);
  f.w2 = packed_dims(d, ff);
  f.head = packed_dims(D.vocab, d);
  return f;
}

size_t fast_packed_bytes(const spec_model_desc &D, int dtype, int L_max) {
  const size_t e = dtype_bytes(dtype), d = D.d_model;
  FastDims f = fast_dims(D);
  size_t per_layer = 4 * al256f(d * e) + al256f(f.qkv.bytes(e)) + al256f(f.o.bytes(e)) + al256f(f.w13.bytes(e)) +
                     al256f(f.w2.bytes(e)) +
                     al256f((size_t)f.qkv.N_pad * 4) + al256f((size_t)f.o.N_pad * 4) + al256f((size_t)f.w13.N_pad * 4) +
                     al256f((size_t)f.w2.N_pad * 4) +
                     al256f((size_t)f.qkv.N_pad * 4) + al256f((size_t)f.w13.N_pad * 4);  // row sums of the packed weights (folded LayerNorm)
  size_t top = 2 * al256f((size_t)f.head.N_pad * 4) + al256f((size_t)D.vocab * d * e) + al256f((size_t)D.max_pos * d * e) + 2 * al256f(d * e) +
               al256f(f.head.bytes(e)) + al256f((size_t)L_max * (d / D.n_heads / 2) * sizeof(float2)) +
               al256f((4 * (size_t)D.n_layers + 1) * sizeof(uint32_t));
  return top + per_layer * (size_t)D.n_layers;
}

static void *bumpf(void *&cursor, size_t bytes) {
  void *p = cursor;
  cursor = (char *)cursor + al256f(bytes);
  return p;
}
static const void *takef(const void *src, size_t bytes, void *&cursor, hipStream_t st) {
  if (!src) return nullptr;
  void *dst = bumpf(cursor, bytes);
  generic_copy(src, dst, bytes, st);
  return dst;
}

bool fast_setup_model(spec_ctx *c, Model &m, const spec_weights *w, void *&cursor, hipStream_t st) {
  const spec_model_desc &D = m.desc;
  const int dt = c->run.dtype;
  const size_t e = dtype_bytes(dt), d = D.d_model;
  const int hd = m.hd;
  FastDims f = fast_dims(D);
  m.p_qkv = f.qkv; m.p_o = f.o; m.p_13 = f.w13; m.p_2 = f.w2; m.p_head = f.head;
  const bool ln = D.norm_kind == SPEC_NORM_LAYER, hb = D.has_bias != 0, swi = D.ffn_kind == SPEC_FFN_SWIGLU;
  // RMS norm: y = W (g * h / rms) = (W diag(g)) h / rms, so the gain goes into the packed weights and the
  // division into the GEMM's epilogue; no norm kernel runs on this path.  LayerNorm the same way with two more
  // terms: W (g * (h - mean) / std + b) = ((W diag(g)) h - mean * rowsum(W diag(g))) / std + W b.
  m.fold_ln = ln;

  m.tok_emb = takef(w->d_tok_emb, (size_t)D.vocab * d * e, cursor, st);
  m.pos_emb = D.pos_kind == SPEC_POS_LEARNED ? takef(w->d_pos_emb, (size_t)D.max_pos * d * e, cursor, st) : nullptr;
  m.final_norm_w = takef(w->d_final_norm_w, d * e, cursor, st);
  m.final_norm_b = ln ? takef(w->d_final_norm_b, d * e, cursor, st) : nullptr;
  // bf16 sources: largest magnitude per matrix -> the power of two its fp16 copy is scaled by
  // (word 4l + {0,1,2,3}: qkv, o, gate-up / fc1, down / fc2 of layer l; the last word: LM head)
  const size_t n_amax = 4 * (size_t)D.n_layers + 1;
  uint32_t *amax = (uint32_t *)bumpf(cursor, n_amax * sizeof(uint32_t));
  generic_zero(amax, n_amax * sizeof(uint32_t), st);
  const bool scaled = dt == SPEC_DTYPE_BF16;
  // with a folded gain the products need the scaling whatever the dtype (fp16 * fp16 may leave the range)
  auto amax_of = [&](size_t word, const void *src, size_t n, const void *gain = nullptr) -> const uint32_t * {
    if (!scaled && !gain) return nullptr;
    launch_absmax(dt, src, n, (int)d, gain, amax + word, st);
    return amax + word;
  };
  void *head = bumpf(cursor, f.head.bytes(e));
  const void *gh = m.final_norm_w;  // the final norm's gain goes into the LM head the same way
  launch_pack_weight(dt, 0, f.head, (int)d, hd, w->d_lm_head, nullptr, nullptr, gh, head,
                     amax_of(n_amax - 1, w->d_lm_head, (size_t)D.vocab * d, gh), st);
  m.lm_head = head;
  if (ln) {
    float *ws_ = (float *)bumpf(cursor, (size_t)f.head.N_pad * 4), *bh = (float *)bumpf(cursor, (size_t)f.head.N_pad * 4);
    generic_zero(bh, (size_t)f.head.N_pad * 4, st);
    launch_fold_ln(dt, 0, f.head, (int)d, hd, w->d_lm_head, nullptr, nullptr, m.final_norm_b, head, ws_, bh, st);
    m.wsum_head = ws_; m.b_head = bh;
  }
  m.rope = nullptr;
  if (D.pos_kind == SPEC_POS_ROPE) {
    float2 *tab = (float2 *)bumpf(cursor, (size_t)c->run.L_max * (hd / 2) * sizeof(float2));
    launch_rope_table(c->run.L_max, hd, D.rope_theta, tab, st);
    m.rope = tab;
  }
  for (int l = 0; l < D.n_layers; ++l) {
    const void *const *T = w->layer_tensors + (size_t)l * SPEC_T_COUNT;
    LayerW &L = m.layers[l];
    L.attn_norm_w = takef(T[SPEC_T_ATTN_NORM_W], d * e, cursor, st);
    L.attn_norm_b = ln ? takef(T[SPEC_T_ATTN_NORM_B], d * e, cursor, st) : nullptr;
    L.ffn_norm_w = takef(T[SPEC_T_FFN_NORM_W], d * e, cursor, st);
    L.ffn_norm_b = ln ? takef(T[SPEC_T_FFN_NORM_B], d * e, cursor, st) : nullptr;
    void *p;
    const size_t a0 = 4 * (size_t)l, ff = D.d_ffn;
    const void *g1 = L.attn_norm_w, *g2 = L.ffn_norm_w;
    p = bumpf(cursor, f.qkv.bytes(e));
    amax_of(a0, T[SPEC_T_WQ], d * d, g1);
    amax_of(a0, T[SPEC_T_WK], d * d, g1);
    launch_pack_weight(dt, 1, f.qkv, (int)d, hd, T[SPEC_T_WQ], T[SPEC_T_WK], T[SPEC_T_WV], g1, p,
                       amax_of(a0, T[SPEC_T_WV], d * d, g1), st);
    L.wqkv = p;
    p = bumpf(cursor, f.o.bytes(e));
    launch_pack_weight(dt, 0, f.o, (int)d, hd, T[SPEC_T_WO], nullptr, nullptr, nullptr, p, amax_of(a0 + 1, T[SPEC_T_WO], d * d), st);
    L.wo = p;
    p = bumpf(cursor, f.w13.bytes(e));
    if (swi) {
      amax_of(a0 + 2, T[SPEC_T_W1], ff * d, g2);
      launch_pack_weight(dt, 2, f.w13, (int)d, hd, T[SPEC_T_W1], T[SPEC_T_W3], nullptr, g2, p,
                         amax_of(a0 + 2, T[SPEC_T_W3], ff * d, g2), st);
    } else {
      launch_pack_weight(dt, 0, f.w13, (int)d, hd, T[SPEC_T_W1], nullptr, nullptr, g2, p,
                         amax_of(a0 + 2, T[SPEC_T_W1], ff * d, g2), st);
    }
    L.w13 = p;
    p = bumpf(cursor, f.w2.bytes(e));
    launch_pack_weight(dt, 0, f.w2, (int)d, hd, T[SPEC_T_W2], nullptr, nullptr, nullptr, p, amax_of(a0 + 3, T[SPEC_T_W2], d * ff), st);
    L.w2 = p;
    L.bqkv = L.bo = L.b13 = L.b2 = nullptr;
    float *fold_bqkv = nullptr, *fold_b13 = nullptr;  // folded LayerNorm: these two GEMMs get a bias whatever the model has
    if (ln && !hb) {
      fold_bqkv = (float *)bumpf(cursor, (size_t)f.qkv.N_pad * 4);
      generic_zero(fold_bqkv, (size_t)f.qkv.N_pad * 4, st);
      fold_b13 = (float *)bumpf(cursor, (size_t)f.w13.N_pad * 4);
      generic_zero(fold_b13, (size_t)f.w13.N_pad * 4, st);
      L.bqkv = fold_bqkv; L.b13 = fold_b13;
    }
    if (hb) {
      float *b = (float *)bumpf(cursor, (size_t)f.qkv.N_pad * 4);
      launch_pack_bias(dt, 1, f.qkv, (int)d, hd, T[SPEC_T_BQ], T[SPEC_T_BK], T[SPEC_T_BV], b, st);
      L.bqkv = b;
      b = (float *)bumpf(cursor, (size_t)f.o.N_pad * 4);
      launch_pack_bias(dt, 0, f.o, (int)d, hd, T[SPEC_T_BO], nullptr, nullptr, b, st);
      L.bo = b;
      if (!swi) {
        b = (float *)bumpf(cursor, (size_t)f.w13.N_pad * 4);
        launch_pack_bias(dt, 0, f.w13, (int)d, hd, T[SPEC_T_B1], nullptr, nullptr, b, st);
        L.b13 = b;
        b = (float *)bumpf(cursor, (size_t)f.w2.N_pad * 4);
        launch_pack_bias(dt, 0, f.w2, (int)d, hd, T[SPEC_T_B2], nullptr, nullptr, b, st);
        L.b2 = b;
      } else if (ln) {
        b = (float *)bumpf(cursor, (size_t)f.w13.N_pad * 4);
        generic_zero(b, (size_t)f.w13.N_pad * 4, st);
        L.b13 = b;
      }
    }
    if (ln) {
      float *ws_ = (float *)bumpf(cursor, (size_t)f.qkv.N_pad * 4);
      launch_fold_ln(dt, 1, f.qkv, (int)d, hd, T[SPEC_T_WQ], T[SPEC_T_WK], T[SPEC_T_WV], L.attn_norm_b, L.wqkv, ws_, (float *)L.bqkv, st);
      L.wsum_qkv = ws_;
      ws_ = (float *)bumpf(cursor, (size_t)f.w13.N_pad * 4);
      if (swi) launch_fold_ln(dt, 2, f.w13, (int)d, hd, T[SPEC_T_W1], T[SPEC_T_W3], nullptr, L.ffn_norm_b, L.w13, ws_, (float *)L.b13, st);
      else launch_fold_ln(dt, 0, f.w13, (int)d, hd, T[SPEC_T_W1], nullptr, nullptr, L.ffn_norm_b, L.w13, ws_, (float *)L.b13, st);
      L.wsum_13 = ws_;
    }
  }
  // the GEMM epilogues undo the scaling: 1 / scale per matrix, from the same words the packing read
  std::vector<uint32_t> h_amax(n_amax, 0u);
  if (hipMemcpyAsync(h_amax.data(), amax, n_amax * sizeof(uint32_t), hipMemcpyDeviceToHost, st) != hipSuccess ||
      hipStreamSynchronize(st) != hipSuccess)
    return false;
  for (int l = 0; l < D.n_layers; ++l) {
    LayerW &L = m.layers[l];
    L.s_qkv = 1.0f / weight_scale(h_amax[4 * l]);
    L.s_o = 1.0f / weight_scale(h_amax[4 * l + 1]);
    L.s_13 = 1.0f / weight_scale(h_amax[4 * l + 2]);
    L.s_2 = 1.0f / weight_scale(h_amax[4 * l + 3]);
  }
  m.s_head = 1.0f / weight_scale(h_amax[n_amax - 1]);
  return true;
}

static GemmArgs base_args(const spec_ctx *c, const PackedDims &p, const void *W, float inv_scale, const void *bias, const void *X, int M) {
  GemmArgs a{};
  a.n_cu = c->n_cu; a.tune = c->gemm_tune; a.sat = c->st.sat;
  a.W = W; a.bias = (const float *)bias; a.X = X; a.out_scale = inv_scale;
  a.M = M; a.N = p.N; a.NT = p.NT; a.KT = p.KT; a.KS = p.KS; a.K_pad = p.K_pad;
  return a;
}

// One pre-norm decoder layer over the M rows of the pass; max_pos is an upper bound of the
// largest row position (sizes the attention grid; chunks past a sequence's end exit at once).
void fast_layer(spec_ctx *c, const Model &m, int layer, int B, int q_rows, int b0, int seq_groups, int max_pos, hipStream_t st) {
  const spec_model_desc &D = m.desc;
  const int dt = c->run.dtype, M = B * q_rows, d = D.d_model;
  const LayerW &L = m.layers[layer];
  Workspace &ws = c->ws;
  const size_t esz = dtype_bytes(dt);
  // the layer's cache area, from batch slot b0 on (a sequence owns H * L_pad * hd elements of each)
  const size_t slot0 = (size_t)b0 * D.n_heads * m.L_pad * m.hd;
  void *kc = (char *)m.kcache + ((size_t)layer * m.kv_area_elems + slot0) * esz;
  void *vc = (char *)m.vcache + ((size_t)layer * m.kv_area_elems + slot0) * esz;

  const bool tgt = &m == &c->tgt;  // only the target model's kernels are timed one by one
  // the norms are folded: ws.x holds fp16(h), left by the producer of h, and the consumer takes 1 / rms (LayerNorm:
  // mean and 1 / std) of its rows from it
  auto consume_norm = [&](GemmArgs &a, const float *wsum) {
    a.fold_x = 1; a.ss_d = d; a.ss_eps = D.norm_eps; a.rinv_ws = ws.row_inv;
    if (m.fold_ln) { a.wsum = wsum; a.mean_ws = ws.row_mean; }
  };
  // the tiled kernel's larger wave tiles read 1 / rms per row from scratch: a small kernel fills it first, unless
  // the producer of the rows has left what is needed
  auto row_inv_first = [&](const GemmArgs &a, int epi) {
    if (c->x_ssq || !gemm_wants_row_inv(a, epi)) return;
    KScope k(c, tgt ? SPEC_KCLASS_NORM : -1);
    launch_row_inv_x(a, st);
  };
  auto produce_norm = [&](GemmArgs &a) {
    a.x_out = ws.x;
    c->x_ssq = gemm_can_leave_ssq(a);  // then the reduction leaves 1 / rms of the new rows where the next GEMM looks for it
    if (c->x_ssq) {
      a.rinv_ws = ws.row_inv; a.ssq_ks = gemm_ks_for(a.N >> 5); a.ss_d = a.N; a.ss_eps = D.norm_eps;
      if (m.fold_ln) a.mean_ws = ws.row_mean;
    }
  };
  {
    GemmArgs a = base_args(c, m.p_qkv, L.wqkv, L.s_qkv, L.bqkv, ws.x, M);
    consume_norm(a, L.wsum_qkv);
    a.q = ws.q; a.kc = kc; a.vc = vc; a.row_pos = ws.row_pos; a.rope = m.rope;
    a.q_rows = q_rows; a.d = d; a.hd = m.hd; a.H = D.n_heads; a.L_pad = m.L_pad; a.seq_groups = seq_groups;
    row_inv_first(a, EPI_QKV);
    KScope k(c, tgt ? SPEC_KCLASS_GEMM_QKV : -1);
    launch_gemm_mfma(dt, a, EPI_QKV, st);
  }
  {
    KScope k(c, tgt ? SPEC_KCLASS_ATTENTION : -1);
    AttnArgs t{};
    t.q = ws.q; t.kc = kc; t.vc = vc; t.row_pos = ws.row_pos; t.out = ws.attn;
    t.part_acc = ws.attn_part; t.part_ml = ws.attn_ml;
    t.B = B; t.q_rows = q_rows; t.H = D.n_heads; t.hd = m.hd; t.L_pad = m.L_pad;
    t.seq_groups = seq_groups;
    t.shape = c->attn_shape;
    t.n_cu = c->n_cu;
    t.NC = std::min(c->NC_max, attn_chunk_of(std::max(max_pos, 0)) + 1);
    launch_attention_mfma(dt, t, st);
  }
  {
    KScope k(c, tgt ? SPEC_KCLASS_GEMM_O : -1);
    GemmArgs a = base_args(c, m.p_o, L.wo, L.s_o, L.bo, ws.attn, M);
    a.h = ws.h; a.part = ws.gemm_part; a.part_rows = (M + 15) / 16 * 16;
    produce_norm(a);
    launch_gemm_mfma(dt, a, EPI_RESIDUAL, st);
  }
  {
    GemmArgs a = base_args(c, m.p_13, L.w13, L.s_13, L.b13, ws.x, M);
    consume_norm(a, L.wsum_13);
    a.act = ws.act; a.f = D.d_ffn;
    const int epi = D.ffn_kind == SPEC_FFN_SWIGLU ? EPI_SWIGLU : EPI_RELU;
    row_inv_first(a, epi);
    KScope k(c, tgt ? SPEC_KCLASS_GEMM_FFN_IN : -1);
    launch_gemm_mfma(dt, a, epi, st);
  }
  {
    KScope k(c, tgt ? SPEC_KCLASS_GEMM_FFN_OUT : -1);
    GemmArgs a = base_args(c, m.p_2, L.w2, L.s_2, L.b2, ws.act, M);
    a.h = ws.h; a.part = ws.gemm_part; a.part_rows = (M + 15) / 16 * 16;
    produce_norm(a);
    launch_gemm_mfma(dt, a, EPI_RESIDUAL, st);
  }
}

// Final norm and LM head with the arg-max fused in, for the rows that need a token: all Mh rows of the pass, or
// (last_of_q > 0) the last row of each of Mh groups of last_of_q rows.
// The final norm is folded into the LM head like the layers' norms (gain in the packed weights, the row statistics
// taken by the GEMM from the fp16 rows the last layer left); the GEMM runs over every row of the pass and the second
// arg-max stage picks the rows that are wanted.
void fast_head(spec_ctx *c, const Model &m, int Mh, int last_of_q, float *logits_or_null, int q, int arg_stride, int32_t *arg_out,
               hipStream_t st) {
  const bool tgt = &m == &c->tgt;
  const int rows = last_of_q > 0 ? Mh * last_of_q : Mh;
  GemmArgs a = base_args(c, m.p_head, m.lm_head, m.s_head, m.fold_ln ? m.b_head : nullptr, c->ws.x, rows);
  a.logits = logits_or_null;
  a.logit_step = last_of_q;  // the head runs over every row of the pass: dump the wanted ones only
  a.part_val = c->ws.head_part;
  a.part_idx = c->ws.head_part_idx;
  a.fold_x = 1; a.ss_d = m.desc.d_model; a.ss_eps = m.desc.norm_eps; a.rinv_ws = c->ws.row_inv;
  if (m.fold_ln) { a.wsum = m.wsum_head; a.mean_ws = c->ws.row_mean; }
  // the row statistics, unless the last layer's down projection has left them
  if (!c->x_ssq && gemm_wants_row_inv(a, EPI_LOGITS)) { KScope k(c, tgt ? SPEC_KCLASS_NORM : -1); launch_row_inv_x(a, st); }
  { KScope k(c, tgt ? SPEC_KCLASS_GEMM_HEAD : -1); launch_gemm_mfma(c->run.dtype, a, EPI_LOGITS, st); }
  { KScope k(c, tgt ? SPEC_KCLASS_OTHER : -1);
    launch_argmax_partials(a.part_val, a.part_idx, Mh, last_of_q, m.p_head.NT, m.desc.vocab, q, arg_stride, arg_out, st); }
}

}  // namespace spec
