// Generic kernels: every dtype (fp32 / bf16 / fp16) and every model shape.  They are the
// path for fp32 runs and for 16-bit shapes the MFMA kernels do not cover.  Plain ALU
// arithmetic in fp32; each output element is reduced in an order fixed by the operand
// shapes alone (never by the number of rows in the pass), so a sequence's tokens do not
// depend on batch size or speculation length.
#include "spec_internal.h"
#include "device_utils.h"
#include <algorithm>

// No implicit fusing of multiplies and adds: which product a compiler folds into an FMA can
// differ between two instantiations of the same source, and results here must be bit-identical
// across launch shapes.  Fused operations are written out with fmaf where they are wanted.
#pragma clang fp contract(off)

namespace spec {

size_t dtype_bytes(int dtype) { return dtype == SPEC_DTYPE_F32 ? 4 : 2; }

// -------------------------------------------------------------------------
__global__ void k_copy_bytes16(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n16; i += stride) dst[i] = src[i];
}
__global__ void k_copy_bytes1(const unsigned char *__restrict__ src, unsigned char *__restrict__ dst, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] = src[i];
}
void generic_copy(const void *src, void *dst, size_t bytes, hipStream_t st) {
  if (!bytes) return;
  if (((uintptr_t)src | (uintptr_t)dst | bytes) % 16 == 0) {
    size_t n16 = bytes / 16;
    unsigned blocks = (unsigned)((n16 + 255) / 256);
    if (blocks > 65535u) blocks = 65535u;
    hipLaunchKernelGGL(k_copy_bytes16, dim3(blocks), dim3(256), 0, st, (const uint4 *)src, (uint4 *)dst, n16);
  } else {
    unsigned blocks = (unsigned)((bytes + 255) / 256);
    if (blocks > 65535u) blocks = 65535u;
    hipLaunchKernelGGL(k_copy_bytes1, dim3(blocks), dim3(256), 0, st, (const unsigned char *)src,
                       (unsigned char *)dst, bytes);
  }
}
__global__ void k_fill_zero(unsigned char *p, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = 0;
}
__global__ void k_fill_zero16(uint4 *p, size_t n16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  const uint4 z = make_uint4(0u, 0u, 0u, 0u);
  for (; i < n16; i += stride) p[i] = z;
}
void generic_zero(void *dst, size_t bytes, hipStream_t st) {
  if (!bytes) return;
  if (((uintptr_t)dst | bytes) % 16 == 0) {
    size_t n16 = bytes / 16;
    unsigned blocks16 = (unsigned)std::min<size_t>((n16 + 255) / 256, 65535);
    hipLaunchKernelGGL(k_fill_zero16, dim3(blocks16), dim3(256), 0, st, (uint4 *)dst, n16);
    return;
  }
  unsigned blocks = (unsigned)((bytes + 255) / 256);
  if (blocks > 65535u) blocks = 65535u;
  hipLaunchKernelGGL(k_fill_zero, dim3(blocks), dim3(256), 0, st, (unsigned char *)dst, bytes);
}

// -------------------------------------------------------------------------
// y[m][n] = sum_k x[m][k] * W[n][k] (+ bias[n]).  One wave per output column n and tile of
// GM rows: lane L accumulates k = L, L+64, ... in ascending order, then a butterfly over
// the lanes.  mode 0: store fp32 into y (row stride ldy); mode 1: add into y (residual).
constexpr int GM = 4;
template <class T>
__global__ void k_gemm_generic(int M, int N, int K, const T *__restrict__ x, const T *__restrict__ W,
                               const T *__restrict__ bias, float *__restrict__ y, int ldy, int mode) {
  const int lane = threadIdx.x & 63;
  const int nn = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  const int m0 = blockIdx.y * GM;
  if (nn >= N) return;
  float acc[GM];
#pragma unroll
  for (int r = 0; r < GM; ++r) acc[r] = 0.f;
  const T *wr = W + (size_t)nn * K;
  for (int k = lane; k < K; k += 64) {
    const float w = Conv<T>::ld(wr, k);
#pragma unroll
    for (int r = 0; r < GM; ++r)
      if (m0 + r < M) acc[r] = fmaf(Conv<T>::ld(x, (size_t)(m0 + r) * K + k), w, acc[r]);
  }
  const float bv = bias ? Conv<T>::ld(bias, nn) : 0.f;
#pragma unroll
  for (int r = 0; r < GM; ++r) {
    float v = wave_sum(acc[r]) + bv;
    if (lane == 0 && m0 + r < M) {
      float *p = y + (size_t)(m0 + r) * ldy + nn;
      *p = mode ? (*p + v) : v;
    }
  }
}

template <class T>
static void gemm_generic(int M, int N, int K, const void *x, const void *W, const void *bias, float *y, int ldy,
                         int mode, hipStream_t st) {
  if (M <= 0) return;
  dim3 grid((N + 3) / 4, (M + GM - 1) / GM);
  hipLaunchKernelGGL(k_gemm_generic<T>, grid, dim3(256), 0, st, M, N, K, (const T *)x, (const T *)W, (const T *)bias,
                     y, ldy, mode);
}

// -------------------------------------------------------------------------
// Rotary embedding on q and k (rotate-half pairing), rounding to the model dtype, and
// the append of this pass's K/V rows at their absolute positions.  One block per
// (row, head); thread i handles pair (i, i + hd/2) and two value elements.
template <class T>
__global__ void k_rope_append(int q_rows, int seq_groups, int H, int hd, int L_pad, int rope, float theta,
                              const float *__restrict__ y /*[M][3d]*/, const int32_t *__restrict__ row_pos,
                              T *__restrict__ qout, T *__restrict__ kc, T *__restrict__ vc) {
  const int m = blockIdx.x, hh = blockIdx.y, b = m / q_rows / seq_groups;  // the row group's sequence
  const int d = H * hd, half = hd >> 1;
  const int pos = row_pos[m];
  const float *yq = y + (size_t)m * 3 * d + (size_t)hh * hd;
  const float *yk = yq + d, *yv = yq + 2 * d;
  for (int i = threadIdx.x; i < half; i += blockDim.x) {
    float c = 1.f, s = 0.f;
    if (rope && pos >= 0) {
      float inv_freq = powf(theta, -2.0f * (float)i / (float)hd);
      sincosf((float)pos * inv_freq, &s, &c);
    }
    float q0 = yq[i], q1 = yq[i + half], k0 = yk[i], k1 = yk[i + half];
    float rq0 = q0 * c - q1 * s, rq1 = q1 * c + q0 * s;
    float rk0 = k0 * c - k1 * s, rk1 = k1 * c + k0 * s;
    T *qr = qout + (size_t)m * d + (size_t)hh * hd;
    Conv<T>::st(qr, 2 * i, rq0);
    Conv<T>::st(qr, 2 * i + 1, rq1);
    if (pos >= 0) {
      size_t ki = kv_k_index(L_pad, H, hd, b, hh, pos, 2 * i);
      Conv<T>::st(kc, ki, rk0);
      Conv<T>::st(kc, ki + 1, rk1);
      Conv<T>::st(vc, kv_v_index(L_pad, H, hd, b, hh, pos, i), yv[i]);
      Conv<T>::st(vc, kv_v_index(L_pad, H, hd, b, hh, pos, i + half), yv[i + half]);
    }
  }
}

// -------------------------------------------------------------------------
// Attention of one query row and one head against keys 0..pos of its sequence (the
// cached prefix plus, causally, the rows of this pass).  One wave per (row, head).
// Scores go to LDS; max, sum and the weighted value sum are taken in ascending key
// order per lane followed by a fixed butterfly, so the result depends on (sequence,
// position) only.
template <class T>
__global__ void k_attn_generic(int q_rows, int seq_groups, int H, int hd, int L_pad, const T *__restrict__ qin,
                               const int32_t *__restrict__ row_pos, const T *__restrict__ kc,
                               const T *__restrict__ vc, T *__restrict__ out) {
  extern __shared__ float sc[];  // [pos+1] scores, then [64][hd] is not needed: values reduced via shuffles
  const int m = blockIdx.x, hh = blockIdx.y, b = m / q_rows / seq_groups, lane = threadIdx.x;
  const int d = H * hd;
  const int pos = row_pos[m];
  T *orow = out + (size_t)m * d + (size_t)hh * hd;
  if (pos < 0) {
    for (int i = lane; i < hd; i += 64) Conv<T>::st(orow, i, 0.f);
    return;
  }
  const int nk = pos + 1;
  const T *qr = qin + (size_t)m * d + (size_t)hh * hd;
  const float scale = 1.0f / sqrtf((float)hd);
  float mx = -INFINITY;
  for (int j = lane; j < nk; j += 64) {
    const T *kr = kc + kv_k_index(L_pad, H, hd, b, hh, j, 0);
    float dot = 0.f;
    for (int i = 0; i < hd; ++i) dot = fmaf(Conv<T>::ld(qr, i), Conv<T>::ld(kr, i), dot);
    dot *= scale;
    sc[j] = dot;
    mx = fmaxf(mx, dot);
  }
  mx = wave_max(mx);
  float sum = 0.f;
  for (int j = lane; j < nk; j += 64) { float p = expf(sc[j] - mx); sc[j] = p; sum += p; }
  sum = wave_sum(sum);
  __syncthreads();
  const float inv = 1.0f / sum;
  for (int i = lane; i < hd; i += 64) {
    float acc = 0.f;
    for (int j = 0; j < nk; ++j) acc = fmaf(sc[j], Conv<T>::ld(vc, kv_v_index(L_pad, H, hd, b, hh, j, i)), acc);
    Conv<T>::st(orow, i, acc * inv);
  }
}

// -------------------------------------------------------------------------
template <class T>
__global__ void k_ffn_act(int M, int f, int swiglu, const float *__restrict__ y, T *__restrict__ act) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)M * f) return;
  size_t m = i / f, c = i % f;
  float r;
  if (swiglu) {
    float g = y[m * 2 * f + c], u = y[m * 2 * f + f + c];
    r = g / (1.0f + expf(-g)) * u;
  } else {
    float v = y[m * f + c];
    r = v > 0.f ? v : 0.f;
  }
  Conv<T>::st(act, i, r);
}

// -------------------------------------------------------------------------
// Weight "packing" for the generic kernels: canonical rows, with q/k/v and gate/up
// concatenated so one GEMM produces them.
static void *bump(void *&cursor, size_t bytes) {
  void *p = cursor;
  cursor = (char *)cursor + ((bytes + 255) & ~(size_t)255);
  return p;
}

size_t generic_packed_bytes(const spec_model_desc &D, int dtype) {
  const size_t e = dtype_bytes(dtype), d = D.d_model, f = D.d_ffn;
  auto al = [](size_t b) { return (b + 255) & ~(size_t)255; };
  const size_t kf = D.ffn_kind == SPEC_FFN_SWIGLU ? 2 : 1;
  size_t per_layer = 4 * al(d * e) + al(3 * d * d * e) + al(3 * d * e) + al(d * d * e) + al(d * e) +
                     al(kf * f * d * e) + al(kf * f * e) + al(d * f * e) + al(d * e);
  size_t top = al((size_t)D.vocab * d * e) * 2 + al((size_t)D.max_pos * d * e) + 2 * al(d * e);
  return top + per_layer * (size_t)D.n_layers;
}

static const void *take(const void *src, size_t bytes, void *&cursor, hipStream_t st) {
  if (!src) return nullptr;
  void *dst = bump(cursor, bytes);
  generic_copy(src, dst, bytes, st);
  return dst;
}

void generic_repack_top(spec_ctx *c, Model &m, const spec_weights *w, void *&cursor, hipStream_t st) {
  const size_t e = dtype_bytes(c->run.dtype), d = m.desc.d_model;
  m.tok_emb = take(w->d_tok_emb, (size_t)m.desc.vocab * d * e, cursor, st);
  m.pos_emb = m.desc.pos_kind == SPEC_POS_LEARNED ? take(w->d_pos_emb, (size_t)m.desc.max_pos * d * e, cursor, st)
                                                  : nullptr;
  m.final_norm_w = take(w->d_final_norm_w, d * e, cursor, st);
  m.final_norm_b = m.desc.norm_kind == SPEC_NORM_LAYER ? take(w->d_final_norm_b, d * e, cursor, st) : nullptr;
  m.lm_head = take(w->d_lm_head, (size_t)m.desc.vocab * d * e, cursor, st);
}

void generic_repack_layer(spec_ctx *c, Model &m, int layer, const spec_weights *w, void *&cursor, hipStream_t st) {
  const size_t e = dtype_bytes(c->run.dtype), d = m.desc.d_model, f = m.desc.d_ffn;
  const void *const *T = w->layer_tensors + (size_t)layer * SPEC_T_COUNT;
  const bool ln = m.desc.norm_kind == SPEC_NORM_LAYER, hb = m.desc.has_bias != 0,
             swi = m.desc.ffn_kind == SPEC_FFN_SWIGLU;
  LayerW &L = m.layers[layer];
  L.attn_norm_w = take(T[SPEC_T_ATTN_NORM_W], d * e, cursor, st);
  L.attn_norm_b = ln ? take(T[SPEC_T_ATTN_NORM_B], d * e, cursor, st) : nullptr;
  L.ffn_norm_w = take(T[SPEC_T_FFN_NORM_W], d * e, cursor, st);
  L.ffn_norm_b = ln ? take(T[SPEC_T_FFN_NORM_B], d * e, cursor, st) : nullptr;
  char *wqkv = (char *)bump(cursor, 3 * d * d * e);
  generic_copy(T[SPEC_T_WQ], wqkv, d * d * e, st);
  generic_copy(T[SPEC_T_WK], wqkv + d * d * e, d * d * e, st);
  generic_copy(T[SPEC_T_WV], wqkv + 2 * d * d * e, d * d * e, st);
  L.wqkv = wqkv;
  L.bqkv = nullptr;
  if (hb) {
    char *bq = (char *)bump(cursor, 3 * d * e);
    generic_copy(T[SPEC_T_BQ], bq, d * e, st);
    generic_copy(T[SPEC_T_BK], bq + d * e, d * e, st);
    generic_copy(T[SPEC_T_BV], bq + 2 * d * e, d * e, st);
    L.bqkv = bq;
  }
  L.wo = take(T[SPEC_T_WO], d * d * e, cursor, st);
  L.bo = hb ? take(T[SPEC_T_BO], d * e, cursor, st) : nullptr;
  if (swi) {
    char *w13 = (char *)bump(cursor, 2 * f * d * e);
    generic_copy(T[SPEC_T_W1], w13, f * d * e, st);
    generic_copy(T[SPEC_T_W3], w13 + f * d * e, f * d * e, st);
    L.w13 = w13;
    L.b13 = nullptr;
    L.w2 = take(T[SPEC_T_W2], d * f * e, cursor, st);
    L.b2 = nullptr;
  } else {
    L.w13 = take(T[SPEC_T_W1], f * d * e, cursor, st);
    L.b13 = hb ? take(T[SPEC_T_B1], f * e, cursor, st) : nullptr;
    L.w2 = take(T[SPEC_T_W2], d * f * e, cursor, st);
    L.b2 = hb ? take(T[SPEC_T_B2], d * e, cursor, st) : nullptr;
  }
}

// -------------------------------------------------------------------------
// One decoder layer over the M rows of the pass (pre-norm residual block).
template <class T>
static void generic_layer_t(spec_ctx *c, const Model &m, int layer, int M, int q_rows, int b0, int seq_groups, hipStream_t st) {
  const spec_model_desc &D = m.desc;
  const int d = D.d_model, f = D.d_ffn, H = D.n_heads, hd = m.hd;
  const LayerW &L = m.layers[layer];
  Workspace &ws = c->ws;
  const size_t esz = sizeof(T);
  const size_t slot0 = (size_t)b0 * H * m.L_pad * hd;  // the pass starts at batch slot b0
  T *kc = (T *)((char *)m.kcache + ((size_t)layer * m.kv_area_elems + slot0) * esz);
  T *vc = (T *)((char *)m.vcache + ((size_t)layer * m.kv_area_elems + slot0) * esz);

  launch_norm(c, m, ws.h, L.attn_norm_w, L.attn_norm_b, ws.x, M, 0, st);
  gemm_generic<T>(M, 3 * d, d, ws.x, L.wqkv, L.bqkv, ws.y32, 3 * d, 0, st);
  hipLaunchKernelGGL(k_rope_append<T>, dim3(M, H), dim3(64), 0, st, q_rows, seq_groups, H, hd, m.L_pad,
                     (int)(D.pos_kind == SPEC_POS_ROPE), D.rope_theta, ws.y32, ws.row_pos, (T *)ws.q, kc, vc);
  hipLaunchKernelGGL(k_attn_generic<T>, dim3(M, H), dim3(64), (size_t)m.L_pad * sizeof(float), st, q_rows, seq_groups, H, hd,
                     m.L_pad, (const T *)ws.q, ws.row_pos, kc, vc, (T *)ws.attn);
  gemm_generic<T>(M, d, d, ws.attn, L.wo, L.bo, ws.h, d, 1, st);

  launch_norm(c, m, ws.h, L.ffn_norm_w, L.ffn_norm_b, ws.x, M, 0, st);
  const bool swi = D.ffn_kind == SPEC_FFN_SWIGLU;
  gemm_generic<T>(M, swi ? 2 * f : f, d, ws.x, L.w13, L.b13, ws.y32, swi ? 2 * f : f, 0, st);
  size_t tot = (size_t)M * f;
  hipLaunchKernelGGL(k_ffn_act<T>, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st, M, f, (int)swi, ws.y32,
                     (T *)ws.act);
  gemm_generic<T>(M, d, f, ws.act, L.w2, L.b2, ws.h, d, 1, st);
}

void generic_layer(spec_ctx *c, const Model &m, int layer, int M, int q_rows, int b0, int seq_groups, hipStream_t st) {
  SPEC_DISPATCH_DTYPE(c->run.dtype, T, generic_layer_t<T>(c, m, layer, M, q_rows, b0, seq_groups, st));
}

// Final norm over the rows that need logits, then the LM head into fp32 logits [Mh][vocab].
void generic_head(spec_ctx *c, const Model &m, int Mh, int last_of_q, float *logits, hipStream_t st) {
  launch_norm(c, m, c->ws.h, m.final_norm_w, m.final_norm_b, c->ws.x, Mh, last_of_q, st);
  SPEC_DISPATCH_DTYPE(c->run.dtype, T,
    gemm_generic<T>(Mh, m.desc.vocab, m.desc.d_model, c->ws.x, m.lm_head, nullptr, logits, m.desc.vocab, 0, st));
}

}  // namespace spec
