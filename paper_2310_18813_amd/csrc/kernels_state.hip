// Kernels that move tokens and per-sequence state: pass assembly + embedding gather,
// norms, arg-max, acceptance/commit, proposal handling, reset/rewind, KV import/export.
#include "spec_internal.h"
#include "device_utils.h"
#include "mfma_tiles.h"

// No implicit fusing of multiplies and adds: which product a compiler folds into an FMA can
// differ between two instantiations of the same source, and results here must be bit-identical
// across launch shapes.  Fused operations are written out with fmaf where they are wanted.
#pragma clang fp contract(off)

namespace spec {

// -------------------------------------------------------------------------
// Row assembly + embedding.  One block per row m = b*q + i.  Decides which token the
// row carries and at which absolute position (pos = -1 marks a dead row: no KV write,
// no attention, logits ignored), then gathers the embedding (plus the learned position
// row for OPT-shape models) into the fp32 residual stream.
// Verification rows follow Alg. 1's call LLM(S, t_1..t_s): pending token, then proposals.
// PREP (models whose RMS norm is folded into the GEMMs): the kernel also leaves what the first layer's QKV GEMM
// consumes, the fp16 copy of the row in fragment order (the GEMM takes 1 / rms of the row from those values).
template <class T, bool PREP>
__global__ __launch_bounds__(256) void k_assemble_embed(int kind, int q, int j, int P, int s_max, int L_max, int vocab, int d,
                                 int learned_pos, int seq_groups, const int32_t *__restrict__ seq, const int32_t *__restrict__ n,
                                 const int32_t *__restrict__ kv_draft, const int32_t *__restrict__ t,
                                 const int32_t *__restrict__ seq_s, const int32_t *__restrict__ P_b,
                                 const T *__restrict__ tok_emb, const T *__restrict__ pos_emb,
                                 int32_t *__restrict__ row_tok, int32_t *__restrict__ row_pos, float *__restrict__ h,
                                 op_t *__restrict__ x, unsigned int *__restrict__ sat) {
  // prefill with several row groups per sequence: group = m / q, sequence = group / seq_groups, and the row's
  // offset from the pass's base position counts the sequence's earlier groups
  const int m = blockIdx.x, grp = m / q;
  const int b = grp / seq_groups, i = (grp % seq_groups) * q + m % q;
  int tok = 0, pos = -1;
  const int nb = n[b];
  // a sequence with its own cap s_b on the speculation length: its rows for proposals beyond s_b are dead
  const int sb = seq_s ? max(0, seq_s[b]) : s_max;
  if (kind == PASS_VERIFY) {
    if (i <= sb) {
      pos = nb - 1 + i;
      tok = (i == 0) ? seq[(size_t)b * L_max + nb - 1] : t[(size_t)b * s_max + i - 1];
    }
  } else if (kind == PASS_DRAFT_FIRST) {
    int p = nb - j - q + i;  // j: positions the pass ends before n_b (catch-up passes of a draft cache far behind)
    if (p >= 0 && p >= kv_draft[b]) { pos = p; tok = seq[(size_t)b * L_max + p]; }
  } else if (kind == PASS_DRAFT_NEXT) {  // draft step j >= 2 yields t_j: wanted only up to s_b
    if (j <= sb) {
      pos = nb + j - 2;
      tok = t[(size_t)b * s_max + j - 2];
    }
  } else {  // PASS_PREFILL: j is the base position
    int p = j + i;
    if (p < P_b[b] - 1) { pos = p; tok = seq[(size_t)b * L_max + p]; }  // the sequence's own prompt length
  }
  if (pos >= L_max) pos = -1;  // cannot happen when the host checks hold; never write out of range
  tok = min(max(tok, 0), vocab - 1);
  if (threadIdx.x == 0) { row_tok[m] = tok; row_pos[m] = pos; }
  float *hr = h + (size_t)m * d;
  auto value = [&](int c) {
    float e = 0.f;
    if (pos >= 0) {
      e = Conv<T>::ld(tok_emb, (size_t)tok * d + c);
      if (learned_pos) e += Conv<T>::ld(pos_emb, (size_t)pos * d + c);
    }
    return e;
  };
  if (!PREP) {
    for (int c = threadIdx.x; c < d; c += blockDim.x) hr[c] = value(c);
    return;
  }
  const int nv = d >> 2;  // four consecutive elements per thread
  for (int c = threadIdx.x; c < nv; c += 256) {
    const float4 o = make_float4(value(4 * c), value(4 * c + 1), value(4 * c + 2), value(4 * c + 3));
    *(float4 *)(hr + 4 * c) = o;
    op_t o4[4] = {to_op_counted(o.x, sat), to_op_counted(o.y, sat), to_op_counted(o.z, sat), to_op_counted(o.w, sat)};
    *(uint2 *)(x + xpack_index(m, 4 * c, d >> 5)) = *(const uint2 *)o4;
  }
}

void launch_assemble_embed(const spec_ctx *c, const Model &m, const PassArgs &pa, hipStream_t st) {
  const int M = pa.B * pa.q;
  const bool prep = m.fast;  // the norms are folded into the GEMMs: they read fp16(h)
  SPEC_DISPATCH_DTYPE(c->run.dtype, T,
    hipLaunchKernelGGL((prep ? k_assemble_embed<T, true> : k_assemble_embed<T, false>), dim3(M), dim3(256), 0, st, (int)pa.kind, pa.q, pa.j, pa.P,
                       c->run.s_max, c->run.L_max, m.desc.vocab, m.desc.d_model,
                       (int)(m.desc.pos_kind == SPEC_POS_LEARNED), pa.seq_groups,
                       c->st.seq + (size_t)pa.b0 * c->run.L_max,
                       c->st.n + pa.b0, c->drf.kv_len ? c->drf.kv_len + pa.b0 : nullptr,
                       c->st.t + (size_t)pa.b0 * c->run.s_max, c->seq_s ? c->seq_s + pa.b0 : nullptr, c->st.P_b + pa.b0,
                       (const T *)m.tok_emb, (const T *)m.pos_emb, c->ws.row_tok, c->ws.row_pos, c->ws.h,
                       (op_t *)c->ws.x, c->st.sat));
}

// -------------------------------------------------------------------------
// RMSNorm / LayerNorm of one row of the fp32 residual stream by a 256-thread workgroup (the models on the generic
// kernels: on the matrix-core path the norms live inside the GEMMs).  Statistics in fp32 with a fixed reduction tree
// (per-thread strided partial, wave butterfly, then the four wave results in order), so a row's result never depends
// on which other rows are in the pass.
__device__ __forceinline__ float block_sum_256(float v, float *sh) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[w] = v;
  __syncthreads();
  return ((sh[0] + sh[1]) + sh[2]) + sh[3];
}

// Row held in registers: thread t owns the float4 groups t, t+256, ... (all loads issued
// before any arithmetic, so the kernel costs one memory round trip, not d/256 of them).
constexpr int NORM_MAX_V4 = 8;  // d <= 8192
// four consecutive parameters (index a multiple of 4) with one load
template <class T>
__device__ __forceinline__ void load4(const T *__restrict__ p, int i, float (&out)[4]) {
  struct alignas(sizeof(T) * 4) Quad { T v[4]; };
  const Quad q = *(const Quad *)(p + i);
#pragma unroll
  for (int k = 0; k < 4; ++k) out[k] = Conv<T>::ld(q.v, k);
}
// the gains and biases of the elements a thread owns (float4 groups t, t + 256, ...); zero where it owns none
template <class T>
__device__ __forceinline__ void norm_params(int kind, int d, const T *__restrict__ gain, const T *__restrict__ bias,
                                            float (&gn)[NORM_MAX_V4][4], float (&bs)[NORM_MAX_V4][4]) {
  const int nv = d >> 2;
#pragma unroll
  for (int i = 0; i < NORM_MAX_V4; ++i) {
    const int c = threadIdx.x + i * 256;
#pragma unroll
    for (int k = 0; k < 4; ++k) { gn[i][k] = 0.f; bs[i][k] = 0.f; }
    if (c < nv) {
      load4(gain, 4 * c, gn[i]);
      if (kind != SPEC_NORM_RMS) load4(bias, 4 * c, bs[i]);
    }
  }
}
// gn, bs: from norm_params, fetched by the caller as early as it can (their latency then passes behind other work)
template <class T>
__device__ __forceinline__ void norm_row(int kind, int d, float eps, const float4 *hr, const float (&gn)[NORM_MAX_V4][4],
                                         const float (&bs)[NORM_MAX_V4][4], int r, void *__restrict__ x, int pack_kt,
                                         unsigned int *__restrict__ sat, float *sh) {
  const int nv = d >> 2;
  float4 v[NORM_MAX_V4];
#pragma unroll
  for (int i = 0; i < NORM_MAX_V4; ++i) {
    const int c = threadIdx.x + i * 256;
    v[i] = c < nv ? hr[c] : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  float mean = 0.f, inv;
  if (kind == SPEC_NORM_RMS) {
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < NORM_MAX_V4; ++i) {
      ss = fmaf(v[i].x, v[i].x, ss); ss = fmaf(v[i].y, v[i].y, ss);
      ss = fmaf(v[i].z, v[i].z, ss); ss = fmaf(v[i].w, v[i].w, ss);
    }
    ss = block_sum_256(ss, sh);
    inv = 1.0f / sqrtf(ss / (float)d + eps);
  } else {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NORM_MAX_V4; ++i) s += (v[i].x + v[i].y) + (v[i].z + v[i].w);
    mean = block_sum_256(s, sh) / (float)d;
    float vs = 0.f;
#pragma unroll
    for (int i = 0; i < NORM_MAX_V4; ++i) {
      const int c = threadIdx.x + i * 256;
      if (c < nv) {
        float a0 = v[i].x - mean, a1 = v[i].y - mean, a2 = v[i].z - mean, a3 = v[i].w - mean;
        vs = fmaf(a0, a0, vs); vs = fmaf(a1, a1, vs); vs = fmaf(a2, a2, vs); vs = fmaf(a3, a3, vs);
      }
    }
    inv = 1.0f / sqrtf(block_sum_256(vs, sh) / (float)d + eps);
  }
#pragma unroll
  for (int i = 0; i < NORM_MAX_V4; ++i) {
    const int c = threadIdx.x + i * 256;
    if (c < nv) {
      const float e[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
      float o[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        o[k] = (e[k] - mean) * inv * gn[i][k];
        if (kind != SPEC_NORM_RMS) o[k] += bs[i][k];
      }
      if (pack_kt > 0) {
        // the consumer is a matrix-core GEMM: fp16 operands, rows stored in fragment order, where four consecutive
        // elements of a row are eight contiguous bytes
        op_t o4[4] = {to_op_counted(o[0], sat), to_op_counted(o[1], sat), to_op_counted(o[2], sat), to_op_counted(o[3], sat)};
        *(uint2 *)((op_t *)x + xpack_index(r, 4 * c, pack_kt)) = *(const uint2 *)o4;
      } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) Conv<T>::st((T *)x, (size_t)r * d + 4 * c + k, o[k]);
      }
    }
  }
}

// -------------------------------------------------------------------------
// RMSNorm / LayerNorm over rows of the fp32 residual stream, output in the model dtype.
// One 256-thread block per output row; statistics in fp32 with a fixed reduction tree
// (per-thread strided partial, wave butterfly, then the four wave results in order), so a
// row's result never depends on which other rows are in the pass.
template <class T>
__global__ __launch_bounds__(256) void k_norm(int kind, int d, float eps, const float *__restrict__ h,
                                              const T *__restrict__ gain, const T *__restrict__ bias,
                                              int last_of_q, void *__restrict__ x,
                                              int pack_kt, unsigned int *__restrict__ sat) {
  __shared__ float sh[4];
  const int r = blockIdx.x;
  // last_of_q > 0: output row r is the last of input rows r * q .. r * q + q - 1 (the rows that need a token)
  const float4 *hr = (const float4 *)(h + (size_t)(last_of_q > 0 ? r * last_of_q + last_of_q - 1 : r) * d);
  // gains and biases are requested first, beside the row, so that their latency passes behind the reductions
  float gn[NORM_MAX_V4][4], bs[NORM_MAX_V4][4];
  norm_params<T>(kind, d, gain, bias, gn, bs);
  norm_row<T>(kind, d, eps, hr, gn, bs, r, x, pack_kt, sat, sh);
}

void launch_norm(const spec_ctx *c, const Model &m, const float *h, const void *gain, const void *bias, void *x,
                 int M, int last_of_q, hipStream_t st) {
  if (M <= 0) return;
  const int pack_kt = m.fast ? m.desc.d_model / 32 : 0;
  SPEC_DISPATCH_DTYPE(c->run.dtype, T,
    hipLaunchKernelGGL(k_norm<T>, dim3(M), dim3(256), 0, st, m.desc.norm_kind, m.desc.d_model, m.desc.norm_eps, h,
                       (const T *)gain, (const T *)bias, last_of_q, x, pack_kt, c->st.sat));
}

// -------------------------------------------------------------------------
// Greedy token per row (Alg. 1 prints "argmin"; Sec. 2 and the caption say the most
// probable token, so arg-max).  Lowest index wins ties.  Row m of the logits goes to
// out[(m / q) * out_stride + m % q].
__global__ void k_argmax_rows(const float *__restrict__ logits, int V, int q, int out_stride, int32_t *__restrict__ out) {
  __shared__ float shv[4];
  __shared__ int shi[4];
  const int m = blockIdx.x;
  const float *row = logits + (size_t)m * V;
  float bv = -INFINITY;
  int bi = 0x7fffffff;
  for (int c = threadIdx.x; c < V; c += 256) argmax_combine(bv, bi, row[c], c);
  wave_argmax(bv, bi);
  if ((threadIdx.x & 63) == 0) { shv[threadIdx.x >> 6] = bv; shi[threadIdx.x >> 6] = bi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) argmax_combine(bv, bi, shv[w], shi[w]);
    if (bi < 0 || bi >= V) bi = 0;
    out[(size_t)(m / q) * out_stride + m % q] = bi;
  }
}

void launch_argmax_rows(const float *logits, int M, int V, int q, int out_stride, int32_t *out, hipStream_t st) {
  if (M <= 0) return;
  hipLaunchKernelGGL(k_argmax_rows, dim3(M), dim3(256), 0, st, logits, V, q, out_stride, out);
}

// -------------------------------------------------------------------------
// -------------------------------------------------------------------------
// External proposals: t_j = table[b][n_b + j - 1] (absolute position), or a plain copy.
__global__ void k_fill_proposals(int B, int s, int s_max, int L_max, const int32_t *__restrict__ table,
                                 const int32_t *__restrict__ n, int32_t *__restrict__ t) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= B * s) return;
  int b = i / s, jj = i % s;
  int p = n[b] + jj;
  t[(size_t)b * s_max + jj] = (p < L_max) ? table[(size_t)b * L_max + p] : 0;
}
void launch_fill_proposals(spec_ctx *c, int s, hipStream_t st) {
  if (s <= 0) return;
  hipLaunchKernelGGL(k_fill_proposals, dim3((c->B * s + 255) / 256), dim3(256), 0, st, c->B, s, c->run.s_max,
                     c->run.L_max, c->prop_table, c->st.n, c->st.t);
}
__global__ void k_copy_proposals(int B, int s, int s_max, const int32_t *__restrict__ src, int32_t *__restrict__ t) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= B * s) return;
  t[(size_t)(i / s) * s_max + i % s] = src[i];
}
void launch_copy_proposals(spec_ctx *c, const int32_t *d_tok, int s, hipStream_t st) {
  if (s <= 0) return;
  hipLaunchKernelGGL(k_copy_proposals, dim3((c->B * s + 255) / 256), dim3(256), 0, st, c->B, s, c->run.s_max, d_tok,
                     c->st.t);
}

// -------------------------------------------------------------------------
// Acceptance + commit, one thread per sequence (Sec. 2, Alg. 1): a proposal survives
// only while all earlier ones matched the target's greedy token; the target's token after
// the last survivor is appended.  Rollback is by length only: the K/V rows written for
// rejected positions stay in the cache and are overwritten by the next round.
// A sequence stops for good after gen_cap[b] emitted tokens: gen_max, or the count at which it emitted the end
// token eos (the tokens a round accepted behind an end token are dropped with it).
__global__ void k_accept(int B, int s, int s_max, int L_max, const int32_t *__restrict__ P_b, int32_t *__restrict__ gen_cap,
                         int eos, int draft_steps, const int32_t *__restrict__ seq_s,
                         const int32_t *__restrict__ t, const int32_t *__restrict__ a, int32_t *__restrict__ seq,
                         int32_t *__restrict__ n, int32_t *__restrict__ kv_draft, int32_t *__restrict__ l_last,
                         unsigned long long *__restrict__ hist, unsigned long long *__restrict__ counters) {
  int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b == 0) atomicAdd(&counters[1], 1ull);
  if (b >= B) return;
  const int n_old = n[b];
  const int gen = n_old - P_b[b];
  const int32_t *tb = t + (size_t)b * s_max;
  const int32_t *ab = a + (size_t)b * (s_max + 1);
  // with a cap per sequence only the first min(s, s_b) proposals were verified, and the draft ran
  // max(1, min(draft_steps, s_b)) live steps for this sequence
  const int sb = seq_s ? min(s, max(0, seq_s[b])) : s;
  if (seq_s && draft_steps > 0) draft_steps = max(1, min(draft_steps, sb));
  int l = 0;
  while (l < sb && tb[l] == ab[l]) ++l;
  const int cap = gen_cap[b];
  int take = min(l + 1, cap - gen);
  if (take < 0) take = 0;
  for (int i = 0; i < take; ++i) {
    const int32_t tok = (i < l) ? tb[i] : ab[l];
    seq[(size_t)b * L_max + n_old + i] = tok;
    if (tok == eos) { take = i + 1; gen_cap[b] = gen + take; }
  }
  const int n_new = n_old + take;
  n[b] = n_new;
  l_last[b] = l;
  if (draft_steps > 0 && kv_draft) {
    int kd = n_old + min(l, draft_steps - 1);
    kv_draft[b] = max(0, min(kd, n_new - 1));
  }
  if (gen < cap) {
    atomicAdd(&hist[l], 1ull);
    atomicAdd(&counters[0], (unsigned long long)take);
  }
}
void launch_accept(spec_ctx *c, int s, hipStream_t st) {
  hipLaunchKernelGGL(k_accept, dim3((c->B + 63) / 64), dim3(64), 0, st, c->B, s, c->run.s_max, c->run.L_max, c->st.P_b,
                     c->st.gen_cap, c->eos, c->draft_j, c->seq_s, c->st.t, c->st.a, c->st.seq, c->st.n, c->drf.kv_len, c->st.l_last,
                     c->st.hist, c->st.counters);
}

// -------------------------------------------------------------------------
// With a prompt: a new batch, every sequence P tokens long — or, ragged, prompt rows of stride P of which sequence
// b uses the first P_b[b] (already on the device).  Without: back to "prompts just given", every sequence to its
// own prompt length.
__global__ void k_state_reset(int B, int P, int ragged, int L_max, int s_max, int gen_max, const int32_t *__restrict__ prompt,
                              int32_t *__restrict__ seq, int32_t *__restrict__ n, int32_t *__restrict__ P_b,
                              int32_t *__restrict__ gen_cap,
                              int32_t *__restrict__ kv_draft,
                              int32_t *__restrict__ l_last, unsigned long long *__restrict__ hist,
                              unsigned long long *__restrict__ counters) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (prompt && i < B * P && (!ragged || i % P < P_b[i / P])) seq[(size_t)(i / P) * L_max + i % P] = prompt[i];
  if (i < B) {
    const int Pi = (prompt && !ragged) ? P : P_b[i];
    P_b[i] = Pi;
    gen_cap[i] = gen_max;
    n[i] = Pi; l_last[i] = 0;
    if (kv_draft) kv_draft[i] = Pi - 1;
  }
  if (i <= s_max) hist[i] = 0ull;
  if (i < 2) counters[i] = 0ull;
}
// One batch slot back to "prompt just given": its tokens, length, draft-cache length.  Counters and the
// accepted-length histogram belong to the whole batch and are left alone.
__global__ void k_state_admit(int P, int gen_max, const int32_t *__restrict__ prompt, int32_t *__restrict__ seq_b,
                              int32_t *__restrict__ n_b, int32_t *__restrict__ P_b_b, int32_t *__restrict__ gen_cap_b,
                              int32_t *__restrict__ kv_draft_b,
                              int32_t *__restrict__ l_last_b) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < P) seq_b[i] = prompt[i];
  if (i == 0) { *n_b = P; *P_b_b = P; *gen_cap_b = gen_max; *l_last_b = 0; if (kv_draft_b) *kv_draft_b = P - 1; }
}
void launch_state_admit(spec_ctx *c, int b, const int32_t *d_prompt, int P, hipStream_t st) {
  hipLaunchKernelGGL(k_state_admit, dim3((P + 255) / 256), dim3(256), 0, st, P, c->run.gen_max, d_prompt,
                     c->st.seq + (size_t)b * c->run.L_max, c->st.n + b, c->st.P_b + b, c->st.gen_cap + b,
                     c->drf.kv_len ? c->drf.kv_len + b : nullptr, c->st.l_last + b);
}
void launch_state_reset(spec_ctx *c, const int32_t *d_prompt, int P_stride, bool ragged, hipStream_t st) {
  int work = c->B * P_stride;
  if (work < c->run.s_max + 1) work = c->run.s_max + 1;
  if (work < 2) work = 2;
  hipLaunchKernelGGL(k_state_reset, dim3((work + 255) / 256), dim3(256), 0, st, c->B, P_stride, (int)ragged, c->run.L_max,
                     c->run.s_max, c->run.gen_max, d_prompt, c->st.seq, c->st.n, c->st.P_b, c->st.gen_cap, c->drf.kv_len, c->st.l_last, c->st.hist,
                     c->st.counters);
}

// -------------------------------------------------------------------------
// KV import / export between the caller's [B][len][d_model] layout and the cache layout
// (keys pair-interleaved inside each head, values blocked by 8 positions).
template <class T>
__global__ void k_kv_convert(int import_, int B, int len, int H, int hd, int L_pad, T *__restrict__ kc,
                             T *__restrict__ vc, T *__restrict__ k_user, T *__restrict__ v_user) {
  const int d = H * hd;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)B * len * d) return;
  int c = (int)(i % d);
  size_t r = i / d;
  int pos = (int)(r % len), b = (int)(r / len);
  int hh = c / hd, e = c % hd;
  size_t ki = kv_k_index(L_pad, H, hd, b, hh, pos, hd_interleave(e, hd));
  size_t vi = kv_v_index(L_pad, H, hd, b, hh, pos, e);
  if (import_) { kc[ki] = k_user[i]; vc[vi] = v_user[i]; }
  else { k_user[i] = kc[ki]; v_user[i] = vc[vi]; }
}
void launch_kv_convert(spec_ctx *c, const Model &m, int layer, int B, int len, void *k, void *v, bool import_,
                       hipStream_t st) {
  size_t total = (size_t)B * len * m.desc.d_model;
  if (!total) return;
  size_t esz = dtype_bytes(c->run.dtype);
  char *kc = (char *)m.kcache + (size_t)layer * m.kv_area_elems * esz;
  char *vc = (char *)m.vcache + (size_t)layer * m.kv_area_elems * esz;
  SPEC_DISPATCH_DTYPE(c->run.dtype, T,
    hipLaunchKernelGGL(k_kv_convert<T>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (int)import_, B, len,
                       m.desc.n_heads, m.hd, m.L_pad, (T *)kc, (T *)vc, (T *)k, (T *)v));
}

}  // namespace spec
